"""Parity of the HIP path (through the C ABI) with the CPU oracle on the same seeded inputs.  Needs an MI355X.

Bars: routing integers (idx, loc, kept, counts, slot_src) bit-exact; encode bit-exact; floating-point outputs within
max-abs-error <= 1e-5 * max|ref| (fp32 storage) or 2e-2 * max|ref| (bf16 storage) of the fp64 oracle.
"""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from paper_2206_03382_amd import synth

pytestmark = pytest.mark.gpu

TOL = {synth.DT_F32: 1e-5, synth.DT_BF16: 2e-2}
RMS_TOL = {synth.DT_F32: 3e-6, synth.DT_BF16: 6e-3}      # tighter, catches small systematic errors


@pytest.fixture(scope="module")
def moe():
    assert torch.cuda.is_available(), "these tests need a GPU"
    from paper_2206_03382_amd import moe as m
    m.lib()                                   # fails loudly if the HIP library is not built
    return m


def dev(a, dtype):
    """numpy fp32 values -> device tensor in the storage dtype (bf16 values are already representable: exact)."""
    if a is None:
        return None
    if dtype == synth.DT_BF16:
        bits = synth.bf16_bits(a)
        return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def host(t):
    return t.float().cpu().numpy() if t.dtype == torch.bfloat16 else t.cpu().numpy()


def assert_close(got, ref, dtype, what):
    ref = np.asarray(ref, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    assert np.isfinite(got).all(), f"{what}: non-finite values"
    scale = np.abs(ref).max()
    err = np.abs(got - ref).max()
    assert err <= TOL[dtype] * scale, f"{what}: max abs err {err:.3e} > {TOL[dtype]:.0e} * max|ref| ({scale:.3e})"
    rms = np.sqrt(np.mean((got - ref) ** 2)) / max(np.sqrt(np.mean(ref ** 2)), 1e-300)
    assert rms <= RMS_TOL[dtype], f"{what}: relative rms err {rms:.3e} > {RMS_TOL[dtype]:.0e}"


def assert_routing_equal(got, ref, C, what=""):
    idx, loc = got["idx"].cpu().numpy(), got["loc"].cpu().numpy()
    assert np.array_equal(idx, ref["idx"]), f"{what} idx differs at {np.argwhere(idx != ref['idx'])[:5]}"
    assert np.array_equal(loc, ref["loc"]), f"{what} loc differs at {np.argwhere(loc != ref['loc'])[:5]}"
    assert np.array_equal(loc < C, ref["kept"])
    assert np.array_equal(got["counts"].cpu().numpy(), ref["counts"])
    np.testing.assert_allclose(got["gate_w"].cpu().numpy(), ref["gate_w"], rtol=1e-5, atol=1e-9)


# ----------------------------------------------------------------------------------------------------------------
# moe_gate_topk from identical fp32 logits
# ----------------------------------------------------------------------------------------------------------------
GATE_CASES = [
    # T, E, k, f, normalize, quantum
    (1, 1, 1, 1.0, 0, 0.0), (5, 1, 1, 1.0, 1, 0.0), (7, 2, 2, 1.0, 1, 0.0), (300, 4, 1, 1.0, 0, 0.0),
    (1000, 5, 3, 1.0, 1, 0.5), (1024, 8, 2, 1.25, 1, 0.0), (777, 12, 12, 0.5, 1, 0.25), (2049, 32, 1, 1.25, 0, 0.0),
    (4096, 64, 2, 1.0, 1, 0.125), (1500, 100, 5, 2.0, 1, 0.0), (3000, 128, 8, 2.0, 1, 0.0), (600, 200, 3, 1.0, 0, 0.5),
    (513, 512, 32, 1.0, 1, 0.0), (256, 16, 4, 8.0, 1, 0.0), (257, 16, 16, 0.1, 1, 1.0),
    (500, 24, 2, 1.0, 1, 0.25), (900, 40, 3, 1.5, 1, 0.0), (700, 17, 17, 1.0, 0, 0.5),     # expert counts that leave lanes of a group partly empty
]


@pytest.mark.parametrize("T,E,k,f,normalize,quantum", GATE_CASES)
def test_gate_topk(moe, T, E, k, f, normalize, quantum):
    logits = synth.make_logits(T, E, seed=T + E + k, quantum=quantum)
    if quantum == 0.0 and E >= 4:
        logits[:, 1] += 0.75                  # an overloaded expert, so that capacity truncation happens
    C = O.capacity(T, E, k, f)
    assert moe.capacity(T, E, k, f) == C
    ref = O.route(logits, k, C, normalize)
    got = moe.gate_topk(torch.from_numpy(logits).cuda(), k, C, normalize)
    assert_routing_equal(got, ref, C, f"T={T} E={E} k={k}")
    assert np.array_equal(got["slot_src"].cpu().numpy(), O.slot_source(ref["idx"], ref["loc"], E, C))
    # all-equal logits: experts 0..k-1 in order, for every token
    flat = moe.gate_topk(torch.zeros((T, E), device="cuda"), k, C, normalize)
    assert np.array_equal(flat["idx"].cpu().numpy(), np.tile(np.arange(k, dtype=np.int32), (T, 1)))


@pytest.mark.parametrize("T,E,k,f,normalize,quantum", GATE_CASES)
def test_gate_topk_batch_prioritized(moe, T, E, k, f, normalize, quantum):
    logits = synth.make_logits(T, E, seed=T + E + k + 100, quantum=quantum)       # quantised logits: many equal priorities
    if quantum == 0.0 and E >= 4:
        logits[:, 1] += 0.75
    C = O.capacity(T, E, k, f)
    ref = O.route(logits, k, C, normalize, bpr=True)
    got = moe.gate_topk(torch.from_numpy(logits).cuda(), k, C, normalize, bpr=True)
    assert_routing_equal(got, ref, C, f"BPR T={T} E={E} k={k}")
    assert np.array_equal(got["slot_src"].cpu().numpy(), O.slot_source(ref["idx"], ref["loc"], E, C))


def test_gate_topk_batch_prioritized_many_tokens(moe):
    """More tokens than one sort tile many times over (and past 2^18): the prioritized order comes from a radix sort, whose
    place computations span several tiles and all three digit passes; quantised logits give long runs of equal priorities."""
    T, E, k = 300001, 16, 2
    logits = synth.make_logits(T, E, seed=77, quantum=0.5)
    C = O.capacity(T, E, k, 0.6)
    ref = O.route(logits, k, C, 1, bpr=True)
    got = moe.gate_topk(torch.from_numpy(logits).cuda(), k, C, 1, bpr=True)
    assert_routing_equal(got, ref, C, "BPR, 300001 tokens")
    assert not np.array_equal(ref["kept"], O.route(logits, k, C, 1)["kept"])       # the order matters at this capacity


def test_gate_topk_is_deterministic(moe):
    logits = torch.from_numpy(synth.make_logits(5000, 64, seed=3, quantum=0.25)).cuda()
    a = moe.gate_topk(logits, 4, 300, 1)
    for _ in range(3):
        b = moe.gate_topk(logits, 4, 300, 1)
        for key in ("idx", "loc", "counts", "slot_src", "gate_w"):
            assert torch.equal(a[key], b[key])


# ----------------------------------------------------------------------------------------------------------------
# moe_gate_route: the gate from the tokens; bf16 gates take the matrix-core logits with exact repair of near-ties
# ----------------------------------------------------------------------------------------------------------------
ROUTE_CASES = [
    # T, M, E, k, f, bias
    (1, 8, 1, 1, 1.0, False), (70, 40, 4, 2, 1.0, True), (1000, 256, 8, 2, 1.25, False), (333, 776, 17, 5, 1.0, True),
    (2048, 1024, 128, 8, 2.0, True), (130, 64, 130, 3, 1.0, False), (65, 2048, 300, 4, 1.5, True), (5000, 264, 64, 2, 1.0, True),
    (3000, 4096, 32, 1, 1.25, False), (777, 136, 40, 40, 1.0, False), (4096, 512, 512, 16, 1.0, True),
]


@pytest.mark.parametrize("dtype", [synth.DT_F32, synth.DT_BF16])
@pytest.mark.parametrize("T,M,E,k,f,bias", ROUTE_CASES)
def test_gate_route(moe, dtype, T, M, E, k, f, bias):
    cfg = synth.CONFIGS[1].scaled(T=T, M=M, H=8, E=E, k=k, dtype=dtype, cfg_id=60 + dtype)
    inp = synth.make_inputs(cfg, seed=T + 1)
    gb = (np.linspace(-1, 1, E).astype(np.float32)) if bias else None
    C = O.capacity(T, E, k, f)
    logits = O.gate_logits(inp["x"], inp["Wg"], gb)
    ref = O.route(logits, k, C, 1)
    got = moe.gate_route(dev(inp["x"], dtype), dev(inp["Wg"], dtype), None if gb is None else torch.from_numpy(gb).cuda(), k, C, 1)
    check_routed_logits(got["logits"].cpu().numpy(), logits)
    assert_routing_equal(got, ref, C, f"gate_route T={T} M={M} E={E} k={k}")
    assert np.array_equal(got["slot_src"].cpu().numpy(), O.slot_source(ref["idx"], ref["loc"], E, C))


@pytest.mark.parametrize("T,M,E,k", [(4096, 512, 16, 2), (3000, 1024, 64, 4), (2500, 256, 128, 8), (1000, 2048, 200, 3)])
def test_gate_route_near_ties(moe, T, M, E, k):
    """Gate weights built to make the matrix-core logits ambiguous: duplicated expert columns (exact ties, which must go
    to the lower index), columns that differ from another in one entry by one bf16 step (true gaps far below the error
    bound of the fast logits), and tokens of all zeros (every logit equal)."""
    cfg = synth.CONFIGS[1].scaled(T=T, M=M, H=8, E=E, k=k, dtype=synth.DT_BF16, cfg_id=62)
    inp = synth.make_inputs(cfg, seed=T + 5)
    x, Wg = inp["x"].copy(), inp["Wg"].copy()
    rng = np.random.default_rng(E)
    for a, b in ((1, 0), (E - 1, 2), (E // 2, 3)):                          # exact duplicates
        Wg[:, a] = Wg[:, b]
    for a, b in ((4, 5), (E - 2, 6), (7, E // 2 + 1)):                      # one entry differs by one bf16 step
        Wg[:, a] = Wg[:, b]
        m = int(rng.integers(0, M))
        bits = synth.bf16_bits(Wg[m:m + 1, a])
        Wg[m, a] = synth.bf16_bits_to_f32(bits + np.uint16(1))[0]
    x[::97] = 0.0
    C = O.capacity(T, E, k, 1.0)
    logits = O.gate_logits(x, Wg, None)
    ref = O.route(logits, k, C, 1)
    d = synth.DT_BF16
    got = moe.gate_route(dev(x, d), dev(Wg, d), None, k, C, 1)
    check_routed_logits(got["logits"].cpu().numpy(), logits)
    assert_routing_equal(got, ref, C, f"near ties T={T} E={E} k={k}")
    # the duplicated columns do occur among the choices, and the lower index comes first whenever both are chosen
    idx = ref["idx"]
    both = (idx == 0).any(axis=1) & (idx == 1).any(axis=1)
    assert both.any()
    assert (np.argmax(idx[both] == 0, axis=1) < np.argmax(idx[both] == 1, axis=1)).all()


# ----------------------------------------------------------------------------------------------------------------
# moe_gate_logits
# ----------------------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [synth.DT_F32, synth.DT_BF16])
@pytest.mark.parametrize("T,M,E,bias", [(1, 8, 1, False), (70, 40, 4, True), (1000, 256, 8, False), (333, 776, 17, True),
                                        (2048, 1024, 128, True), (130, 64, 130, False), (65, 2048, 300, True)])
def test_gate_logits(moe, dtype, T, M, E, bias):
    cfg = synth.CONFIGS[1].scaled(T=T, M=M, H=8, E=E, dtype=dtype, cfg_id=40 + dtype)
    inp = synth.make_inputs(cfg, seed=T)
    gb = (np.linspace(-1, 1, E).astype(np.float32)) if bias else None
    ref = O.gate_logits(inp["x"], inp["Wg"], gb)
    got = moe.gate_logits(dev(inp["x"], dtype), dev(inp["Wg"], dtype), None if gb is None else torch.from_numpy(gb).cuda())
    got = got.cpu().numpy()
    # fp64 accumulation on both sides, one rounding to fp32: equal except where the fp64 sums straddle a rounding
    # boundary (last bit, rare)
    ulp = np.spacing(np.abs(ref).astype(np.float32))
    assert (np.abs(got - ref) <= ulp).all()
    assert (got != ref).mean() <= 1e-4


# ----------------------------------------------------------------------------------------------------------------
# cosine router front-end (moe_gate_logits_cosine) followed by the usual top-k
# ----------------------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,T,M,D,E,k,tau", [
    (synth.DT_BF16, 1000, 64, 256, 8, 2, 0.07), (synth.DT_F32, 777, 40, 48, 100, 3, 0.5), (synth.DT_BF16, 2048, 256, 256, 130, 4, 0.005),
    (synth.DT_F32, 1, 8, 1, 1, 1, 1.0), (synth.DT_BF16, 300, 128, 70, 64, 1, 0.01)])
def test_cosine_router(moe, dtype, T, M, D, E, k, tau):
    cfg = synth.CONFIGS[1].scaled(T=T, M=M, H=8, E=max(E, k), k=k, dtype=dtype, cfg_id=48)
    x = synth.make_inputs(cfg, seed=T)["x"]
    rng = np.random.default_rng(T + D)
    Wp = (rng.standard_normal((M, D)) / np.sqrt(M)).astype(np.float32)
    if dtype == synth.DT_BF16:
        Wp = synth.round_to_bf16(Wp)
    Me = rng.standard_normal((E, D)).astype(np.float32)
    ref = O.cosine_gate_logits(x, Wp, Me, tau)
    got = moe.gate_logits_cosine(dev(x, dtype), dev(Wp, dtype), torch.from_numpy(Me).cuda(), tau)
    g = got.cpu().numpy()
    ulp = np.spacing(np.abs(ref).astype(np.float32))
    assert (np.abs(g - ref) <= ulp).all() and (g != ref).mean() <= max(1e-4, 1.5 / g.size)
    C = O.capacity(T, E, k, 1.25)
    r = O.route(ref, k, C, 1)
    assert_routing_equal(moe.gate_topk(got, k, C, 1), r, C, "cosine router")


# ----------------------------------------------------------------------------------------------------------------
# moe_encode / moe_decode
# ----------------------------------------------------------------------------------------------------------------
DISPATCH_CASES = [(1, 8, 1, 1, 1.0), (50, 24, 3, 2, 0.7), (1000, 256, 8, 2, 1.25), (777, 776, 5, 3, 0.5), (2049, 1536, 32, 1, 1.25),
                  (1500, 4096, 16, 8, 2.0), (64, 8200, 4, 2, 1.0)]


@pytest.mark.parametrize("dtype", [synth.DT_F32, synth.DT_BF16])
@pytest.mark.parametrize("T,M,E,k,f", DISPATCH_CASES)
def test_encode_decode(moe, dtype, T, M, E, k, f):
    cfg = synth.CONFIGS[1].scaled(T=T, M=M, H=8, E=E, k=k, f=f, dtype=dtype, cfg_id=42)
    x = synth.make_inputs(cfg, seed=M)["x"]
    logits = synth.make_logits(T, E, seed=T, quantum=0.25)
    C = O.capacity(T, E, k, f)
    r = O.route(logits, k, C, 1)
    g = moe.gate_topk(torch.from_numpy(logits).cuda(), k, C, 1)
    xd = dev(x, dtype)
    Zref = O.encode_sparse(x, r["idx"], r["loc"], E, C, dtype=np.float32)
    for slot_src in (g["slot_src"], None):                       # gather form, scatter form
        Z = moe.encode(xd, g["idx"], g["loc"], slot_src, E, C)
        assert np.array_equal(host(Z).view(np.uint32), Zref.view(np.uint32)), "encode must be a bit-exact copy / +0 fill"
    Y = synth.make_inputs(cfg.scaled(T=E * C, cfg_id=43), seed=7)["x"].reshape(E, C, M)     # stands in for expert outputs
    ref = O.decode_sparse(Y, r["idx"], r["loc"], r["gate_w"], C)
    out = host(moe.decode(dev(Y, dtype), g["idx"], g["loc"], g["gate_w"]))
    assert_close(out, ref, dtype, "decode")
    dead = (~r["kept"]).all(axis=1)
    assert (out[dead].view(np.uint32) == 0).all(), "all-dropped tokens must be exact +0 rows"


# ----------------------------------------------------------------------------------------------------------------
# backward of encode / decode (the differentiable fast encode and decode operators)
# ----------------------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [synth.DT_F32, synth.DT_BF16])
@pytest.mark.parametrize("T,M,E,k,f", DISPATCH_CASES)
def test_encode_decode_backward(moe, dtype, T, M, E, k, f):
    cfg = synth.CONFIGS[1].scaled(T=T, M=M, H=8, E=E, k=k, f=f, dtype=dtype, cfg_id=44)
    logits = synth.make_logits(T, E, seed=T + 1, quantum=0.25)
    C = O.capacity(T, E, k, f)
    r = O.route(logits, k, C, 1)
    g = moe.gate_topk(torch.from_numpy(logits).cuda(), k, C, 1)
    assert_routing_equal(g, r, C)
    d_out = synth.make_inputs(cfg, seed=M + 1)["x"]                                            # stands in for d(out)
    slabs = synth.make_inputs(cfg.scaled(T=E * C, cfg_id=45), seed=8)["x"].reshape(E, C, M)   # stands in for dZ and for Y
    # encode backward: sum of a token's kept slot rows; dead tokens get exact +0
    dx = host(moe.encode_backward(dev(slabs, dtype), g["idx"], g["loc"]))
    assert_close(dx, O.encode_backward_sparse(slabs, r["idx"], r["loc"], C), dtype, "encode backward")
    dead = (~r["kept"]).all(axis=1)
    assert (dx[dead].view(np.uint32) == 0).all()
    # decode backward: weighted rows into the slots (unfilled slots exact +0), and the gate-weight gradient
    dY, dgw = moe.decode_backward(dev(d_out, dtype), dev(slabs, dtype), g["idx"], g["loc"], g["gate_w"], g["slot_src"])
    dY, dgw = host(dY), dgw.cpu().numpy()
    # the oracle takes the gate weights it computed itself (fp64); the device's fp32 weights differ by rounding only
    assert_close(dY, O.decode_backward_sparse(d_out, r["idx"], r["loc"], r["gate_w"], E, C), dtype, "decode backward, dY")
    unfilled = O.slot_source(r["idx"], r["loc"], E, C) < 0
    assert (dY[unfilled].view(np.uint32) == 0).all()
    ref = O.gate_weight_grad(d_out, slabs, r["idx"], r["loc"], C)
    scale = 0.0                                                # size of the sums: the largest sum of |terms| of a kept choice
    for j in range(k):
        t = np.nonzero(r["kept"][:, j])[0]
        if len(t):
            scale = max(scale, float(np.abs(d_out[t].astype(np.float64) * slabs[r["idx"][t, j], r["loc"][t, j]]).sum(axis=1).max()))
    assert np.abs(dgw - ref).max() <= 1e-5 * max(scale, 1e-30), "gate-weight gradient"
    assert (dgw[~r["kept"]] == 0).all()


# ----------------------------------------------------------------------------------------------------------------
# moe_expert_ffn
# ----------------------------------------------------------------------------------------------------------------
FFN_CASES = [
    # dtype, E, C, M, H, act, bias, use_counts
    (synth.DT_F32, 1, 1, 8, 8, O.ACT_RELU, False, False),
    (synth.DT_F32, 3, 70, 40, 72, O.ACT_GELU, True, True),
    (synth.DT_F32, 4, 256, 256, 512, O.ACT_RELU, False, False),
    (synth.DT_F32, 2, 130, 264, 136, O.ACT_SILU, True, True),
    (synth.DT_BF16, 2, 100, 72, 40, O.ACT_GELU, True, True),            # generic (non-MFMA) bf16 shapes
    (synth.DT_BF16, 3, 300, 256, 256, O.ACT_RELU, False, False),        # MFMA path, ragged last row tile
    (synth.DT_BF16, 2, 513, 512, 768, O.ACT_GELU, True, True),
    (synth.DT_BF16, 5, 1000, 768, 1024, O.ACT_SILU, True, True),
    (synth.DT_BF16, 1, 256, 1024, 256, O.ACT_GELU, False, False),
    (synth.DT_BF16, 9, 37, 256, 512, O.ACT_SILU, False, True),
]


@pytest.mark.parametrize("dtype,E,C,M,H,act,bias,use_counts", FFN_CASES)
def test_expert_ffn(moe, dtype, E, C, M, H, act, bias, use_counts):
    cfg = synth.CONFIGS[1].scaled(T=E * C, M=M, H=H, E=E, dtype=dtype, cfg_id=44)
    inp = synth.make_inputs(cfg, seed=C, bias_std=0.5 if bias else 0.0)
    Z = inp["x"].reshape(E, C, M)
    counts = None
    if use_counts:
        counts = np.random.default_rng(C).integers(0, C + 40, size=E).astype(np.int32)   # some empty, some beyond C
        counts[0] = C // 2
        if E > 1:
            counts[1] = 0
    ref = O.expert_ffn(Z, inp["W1"], inp["b1"], inp["W2"], inp["b2"], act, rows=counts)
    Yd = torch.full((E, C, M), float("nan"), device="cuda").to(torch.bfloat16 if dtype == synth.DT_BF16 else torch.float32)
    moe.expert_ffn(dev(Z, dtype), dev(inp["W1"], dtype), dev(inp["b1"], dtype), dev(inp["W2"], dtype), dev(inp["b2"], dtype), act,
                   None if counts is None else torch.from_numpy(counts).cuda(), Y=Yd)
    got = host(Yd)
    if counts is None:
        assert_close(got, ref, dtype, "ffn")
    else:
        rows = np.minimum(counts, C)
        mask = np.arange(C)[None, :] < rows[:, None]
        assert_close(got[mask], ref[mask], dtype, "ffn (filled rows)")
        assert np.isnan(got[~mask]).all(), "rows past counts[e] must be left untouched"


# The grouped GEMM deals its live tiles to the XCDs in groups of 32, 16 or 8, chosen on the device from the number of
# live tiles (below 512: 8; below 1024: 16): fills that put the first product exactly at, just below and between the
# thresholds, with ragged last row tiles and an empty expert.  H = 1024 gives the first product
# four column tiles per row tile and the second one.
@pytest.mark.parametrize("row_tiles", [127, 128, 200, 255, 256])
def test_expert_ffn_tile_group_sizes(moe, row_tiles):
    dtype, E, M, H, act = synth.DT_BF16, 6, 256, 1024, O.ACT_SILU
    tiles = np.array([row_tiles - 3 * (row_tiles // 4) - 1, row_tiles // 4, 0, row_tiles // 4, 1, row_tiles // 4])   # per expert
    assert tiles.sum() == row_tiles and (tiles >= 0).all()
    ragged = np.array([-37, 0, 0, -255, -200, 0])                    # rows short of a whole last tile
    counts = (tiles * 256 + np.where(tiles > 0, ragged, 0)).astype(np.int32)
    C = int(counts.max())
    live = int(((counts + 255) // 256).sum())
    assert live == row_tiles
    cfg = synth.CONFIGS[1].scaled(T=E * C, M=M, H=H, E=E, dtype=dtype, cfg_id=45)
    inp = synth.make_inputs(cfg, seed=row_tiles, bias_std=0.5)
    Z = inp["x"].reshape(E, C, M)
    ref = O.expert_ffn(Z, inp["W1"], inp["b1"], inp["W2"], inp["b2"], act, rows=counts)
    Yd = torch.full((E, C, M), float("nan"), device="cuda").to(torch.bfloat16)
    moe.expert_ffn(dev(Z, dtype), dev(inp["W1"], dtype), dev(inp["b1"], dtype), dev(inp["W2"], dtype), dev(inp["b2"], dtype), act,
                   torch.from_numpy(counts).cuda(), Y=Yd)
    got = host(Yd)
    rows = np.minimum(counts, C)
    mask = np.arange(C)[None, :] < rows[:, None]
    assert_close(got[mask], ref[mask], dtype, "ffn (filled rows)")
    assert np.isnan(got[~mask]).all(), "rows past counts[e] must be left untouched"


def test_expert_ffn_gelu_epilogue_range(moe):
    """The matrix-core GEMM's GeLU epilogue through the kernel itself: one expert whose first layer is 6 x identity on
    inputs spanning [-1, 1] (so the pre-activations span [-6, 6], each an exact bf16 product) and whose second layer
    is the identity, so that Y = gelu(6 z) element by element."""
    C, M = 512, 256
    z = synth.round_to_bf16(np.linspace(-1.0, 1.0, C * M, dtype=np.float32).reshape(1, C, M))
    eye6 = (6.0 * np.eye(M, dtype=np.float32))[None]
    eye = np.eye(M, dtype=np.float32)[None]
    ref = O.expert_ffn(z, eye6, None, eye, None, O.ACT_GELU)
    pre = 6.0 * z.astype(np.float64)
    assert pre.min() <= -5.9 and pre.max() >= 5.9
    Y = host(moe.expert_ffn(dev(z, synth.DT_BF16), dev(eye6, synth.DT_BF16), None, dev(eye, synth.DT_BF16), None, O.ACT_GELU))
    # the hidden value and the output are each rounded to bf16 once: two half-ulp roundings of |value| <= 6
    assert np.abs(Y - ref).max() <= 2.0 ** -8 * np.maximum(np.abs(ref), 2.0 ** -126).max()
    assert (np.abs(Y - ref) <= 2.0 ** -7 * np.abs(ref) + 1e-6).all()


# ----------------------------------------------------------------------------------------------------------------
# moe_gate_backward
# ----------------------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [synth.DT_F32, synth.DT_BF16])
@pytest.mark.parametrize("T,M,E,k,normalize", [(1, 8, 1, 1, 1), (70, 40, 4, 2, 1), (1000, 256, 8, 2, 1), (333, 776, 17, 5, 0),
                                               (2500, 128, 128, 8, 1), (1025, 64, 300, 3, 1), (20000, 256, 64, 2, 1),
                                               (900, 64, 24, 3, 0), (3000, 512, 128, 4, 1), (777, 256, 64, 2, 0),
                                               (1500, 256, 40, 3, 1), (600, 512, 100, 5, 0)])
def test_gate_backward(moe, dtype, T, M, E, k, normalize):
    cfg = synth.CONFIGS[1].scaled(T=T, M=M, H=8, E=E, k=k, dtype=dtype, cfg_id=50)
    inp = synth.make_inputs(cfg, seed=T + 3)
    x, Wg = inp["x"], inp["Wg"]
    logits = O.gate_logits(x, Wg, None)
    idx = O.topk_experts(logits, k)
    rng = np.random.default_rng(T + E)
    dgw = rng.standard_normal((T, k)).astype(np.float32)
    base = synth.make_inputs(cfg.scaled(cfg_id=51), seed=T + 4)["x"]               # stands in for the dispatch path's dx
    ref_dl = O.gate_backward(logits, idx, dgw, normalize)
    ref = O.gate_logits_backward(x, Wg, ref_dl)
    dxd = dev(base, dtype).clone()
    g = moe.gate_backward(dev(x, dtype), dev(Wg, dtype), torch.from_numpy(logits).cuda(), torch.from_numpy(idx).cuda(),
                          torch.from_numpy(dgw).cuda(), normalize, dx=dxd)
    torch.cuda.synchronize()
    dl = g["dlogits"].cpu().numpy()
    assert np.abs(dl - ref_dl).max() <= 1e-5 * max(np.abs(ref_dl).max(), 1e-30)
    assert_close(host(g["dx"]), base.astype(np.float64) + ref["dx"], dtype, "gate dx (accumulated)")
    # the gate's own term, without a base to hide behind: a call that does not accumulate, scaled by the term itself
    g0 = moe.gate_backward(dev(x, dtype), dev(Wg, dtype), torch.from_numpy(logits).cuda(), torch.from_numpy(idx).cuda(),
                           torch.from_numpy(dgw).cuda(), normalize)
    assert_close(host(g0["dx"]), ref["dx"], dtype, "gate dx (not accumulated)")
    assert_close(host(g["dWg"]), ref["dWg"], dtype, "dWg")
    assert np.abs(g["dbias"].cpu().numpy() - ref["dbias"]).max() <= 1e-5 * max(np.abs(ref_dl).sum(axis=0).max(), 1e-30)


# ----------------------------------------------------------------------------------------------------------------
# moe_expert_ffn_backward
# ----------------------------------------------------------------------------------------------------------------
FFN_BWD_CASES = [
    # dtype, E, C, M, H, act, bias, use_counts
    (synth.DT_F32, 1, 1, 8, 8, O.ACT_RELU, False, False),
    (synth.DT_F32, 3, 70, 40, 72, O.ACT_GELU, True, True),
    (synth.DT_F32, 2, 130, 264, 136, O.ACT_SILU, True, True),
    (synth.DT_BF16, 2, 100, 72, 40, O.ACT_GELU, True, True),            # generic (non-MFMA) bf16 shapes
    (synth.DT_BF16, 3, 300, 256, 256, O.ACT_RELU, False, False),        # MFMA GEMMs, capacity not a multiple of 64
    (synth.DT_BF16, 2, 513, 512, 768, O.ACT_GELU, True, True),
    (synth.DT_BF16, 5, 1000, 768, 1024, O.ACT_SILU, True, True),
    (synth.DT_BF16, 9, 37, 256, 512, O.ACT_SILU, False, True),
]


@pytest.mark.parametrize("dtype,E,C,M,H,act,bias,use_counts", FFN_BWD_CASES)
def test_expert_ffn_backward(moe, dtype, E, C, M, H, act, bias, use_counts):
    cfg = synth.CONFIGS[1].scaled(T=E * C, M=M, H=H, E=E, dtype=dtype, act=act, cfg_id=46)
    inp = synth.make_inputs(cfg, seed=C + 1, bias_std=0.25 if bias else 0.0)
    Z = inp["x"].reshape(E, C, M)
    dY = synth.make_inputs(cfg.scaled(cfg_id=47), seed=C + 2)["x"].reshape(E, C, M)
    rows = None
    if use_counts:
        rows = np.array([(7 * e * C // (2 * max(E - 1, 1)) + (e % 3)) % (C + 3) for e in range(E)], dtype=np.int32)   # 0 .. above C
    ref = O.expert_ffn_backward(Z, inp["W1"], inp["b1"], inp["W2"], dY, act, rows=rows)
    Zd, W1, b1, W2, b2 = dev(Z, dtype), dev(inp["W1"], dtype), dev(inp["b1"], dtype), dev(inp["W2"], dtype), dev(inp["b2"], dtype)
    counts = None if rows is None else torch.from_numpy(rows).cuda()
    hidden = torch.empty((E, C, H), dtype=Zd.dtype, device="cuda")
    Y = moe.expert_ffn(Zd, W1, b1, W2, b2, act, counts=counts, hidden=hidden)
    g = moe.expert_ffn_backward(Zd, W1, b1, W2, hidden, dev(dY, dtype), act, counts=counts)
    # the training forward keeps the pre-activations: same hidden and Y, and the same gradients as with the recompute
    Yt, hidden_t, pre = moe.expert_ffn_train(Zd, W1, b1, W2, b2, act, counts=counts)
    gs = moe.expert_ffn_backward(Zd, W1, b1, W2, hidden_t, dev(dY, dtype), act, counts=counts, pre=pre)
    torch.cuda.synchronize()
    live = np.zeros((E, C), dtype=bool)
    for e in range(E):
        live[e, :C if rows is None else min(max(int(rows[e]), 0), C)] = True
    lv = torch.from_numpy(live).cuda()
    assert torch.equal(Yt[lv], Y[lv]) and torch.equal(hidden_t[lv], hidden[lv])
    if live.any():
        ref_pre = np.einsum("ecm,emh->ech", Z.astype(np.float64), inp["W1"].astype(np.float64))
        if inp["b1"] is not None:
            ref_pre = ref_pre + inp["b1"].astype(np.float64)[:, None, :]
        assert_close(host(pre)[live], ref_pre[live], dtype, "pre-activations")
    for name in ("dZ", "dW1", "db1", "dW2", "db2"):
        a, b = gs[name], g[name]
        assert torch.equal(a[lv], b[lv]) if name == "dZ" else torch.equal(a, b), name
    if live.any():
        assert_close(host(g["dZ"])[live], ref["dZ"][live], dtype, "dZ")
    for name in ("dW1", "db1", "dW2", "db2"):
        got = host(g[name])
        if np.abs(ref[name]).max() == 0:
            assert (got == 0).all(), name
        else:
            assert_close(got, ref[name], dtype, name)


# ----------------------------------------------------------------------------------------------------------------
# moe_layer_forward: reduced versions of the five workloads (several tiles + ragged tails), full element-wise check
# ----------------------------------------------------------------------------------------------------------------
def run_layer(moe, cfg, inp):
    d = cfg.dtype
    layer = moe.MoELayer(dev(inp["Wg"], d), None if inp["gate_bias"] is None else torch.from_numpy(inp["gate_bias"]).cuda(),
                         dev(inp["W1"], d), dev(inp["b1"], d), dev(inp["W2"], d), dev(inp["b2"], d),
                         T=cfg.T, k=cfg.k, f=cfg.f, normalize=cfg.normalize, act=cfg.act, keep_routing=True)
    out = layer.forward(dev(inp["x"], d))
    torch.cuda.synchronize()
    return layer, out


def check_logits(got, ref, floor=0.0):
    """Exactly rounded logits (fp64 sums on both sides): equal up to the last bit, in all but a few entries."""
    ulp = np.spacing(np.abs(ref).astype(np.float32))
    assert (np.abs(got - ref) <= ulp).all() and (got != ref).mean() <= max(1e-4, floor / got.size)


def check_routed_logits(got, ref):
    """Logits as the gate stores them inside the layer: exactly rounded where a decision needed them, within the
    matrix-core path's error bound elsewhere; the bar for floating-point values, 1e-5 * max|ref|."""
    assert np.abs(got - ref).max() <= 1e-5 * np.abs(ref).max()


SMALL_LAYERS = [
    synth.CONFIGS[0].scaled(T=300, M=40, H=72, E=3),
    synth.CONFIGS[0],
    synth.CONFIGS[1].scaled(T=1500, M=256, H=512, E=8),
    synth.CONFIGS[1].scaled(T=2000, M=264, H=520, E=8),                   # shapes that take the generic bf16 GEMM
    synth.CONFIGS[2].scaled(T=1960, M=768, H=1024, E=32),
    synth.CONFIGS[3].scaled(T=4096, M=256, H=512, E=64),
    synth.CONFIGS[4].scaled(T=4096, M=512, H=256, E=128),
]


@pytest.mark.parametrize("cfg", SMALL_LAYERS, ids=lambda c: f"{c.name}-T{c.T}-M{c.M}-H{c.H}-E{c.E}")
@pytest.mark.parametrize("bias", [False, True])
def test_layer_small(moe, cfg, bias):
    inp = synth.make_inputs(cfg, seed=0, bias_std=0.25 if bias else 0.0)
    tier = "dense" if cfg.T * cfg.E * O.capacity(cfg.T, cfg.E, cfg.k, cfg.f) <= 2 ** 28 else "sparse"
    ref = O.moe_layer(inp["x"], inp["Wg"], inp["gate_bias"], inp["W1"], inp["b1"], inp["W2"], inp["b2"],
                      cfg.k, cfg.f, cfg.normalize, cfg.act, tier=tier)
    layer, out = run_layer(moe, cfg, inp)
    assert layer.C == ref["C"]
    check_routed_logits(layer.routing["logits"].cpu().numpy(), ref["logits"])
    assert_routing_equal(layer.routing, ref, ref["C"], cfg.name)
    got = host(out)
    assert_close(got, ref["out"], cfg.dtype, f"layer output ({cfg.name})")
    dead = (~ref["kept"]).all(axis=1)
    assert (got[dead].view(np.uint32) == 0).all()


# ----------------------------------------------------------------------------------------------------------------
# forward + backward of the whole layer through the separate entry points
# ----------------------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("cfg", [synth.CONFIGS[0].scaled(T=300, M=40, H=72, E=3), synth.CONFIGS[1].scaled(T=1500, M=256, H=512, E=8),
                                 synth.CONFIGS[3].scaled(T=4096, M=256, H=512, E=64)], ids=lambda c: f"{c.name}-T{c.T}-E{c.E}")
def test_layer_forward_backward(moe, cfg):
    inp = synth.make_inputs(cfg, seed=11, bias_std=0.25)
    d_out = synth.make_inputs(cfg.scaled(cfg_id=52), seed=12)["x"]
    ref = O.moe_layer_backward(inp["x"], inp["Wg"], inp["gate_bias"], inp["W1"], inp["b1"], inp["W2"], inp["b2"],
                               cfg.k, cfg.f, cfg.normalize, cfg.act, d_out)
    d = cfg.dtype
    gb = None if inp["gate_bias"] is None else torch.from_numpy(inp["gate_bias"]).cuda()
    got = moe.layer_forward_backward(dev(inp["x"], d), dev(inp["Wg"], d), gb, dev(inp["W1"], d), dev(inp["b1"], d),
                                     dev(inp["W2"], d), dev(inp["b2"], d), cfg.k, cfg.f, cfg.normalize, cfg.act, dev(d_out, d))
    torch.cuda.synchronize()
    assert_routing_equal(got["routing"], ref["forward"], ref["forward"]["C"], cfg.name)
    assert_close(host(got["out"]), ref["forward"]["out"], d, "out")
    for name in ("dx", "dWg", "dW1", "db1", "dW2", "db2"):
        assert_close(host(got[name]), ref[name], d, name)
    scale = np.abs(ref["dgate_bias"]).max()
    assert np.abs(got["dgate_bias"].cpu().numpy() - ref["dgate_bias"]).max() <= (1e-4 if d == synth.DT_F32 else 2e-2) * max(scale, 1e-30)
    # the same step through the two layer-level entry points (one state buffer, no allocation in between): run twice
    # on the same state; same kernels in the same order, so every result is bit-identical to the composed path
    tl = moe.TrainLayer(dev(inp["Wg"], d), gb, dev(inp["W1"], d), dev(inp["b1"], d), dev(inp["W2"], d), dev(inp["b2"], d),
                        T=cfg.T, k=cfg.k, f=cfg.f, normalize=cfg.normalize, act=cfg.act)
    xd, dod = dev(inp["x"], d), dev(d_out, d)
    for _ in range(2):
        out2 = tl.forward(xd)
        g2 = tl.backward(xd, dod)
        torch.cuda.synchronize()
        assert torch.equal(out2, got["out"])
        for name in ("dx", "dWg", "dgate_bias", "dW1", "db1", "dW2", "db2"):
            assert torch.equal(g2[name], got[name]), name


# The training step reads the experts' input rows through the slot -> token map (no dispatch buffer).  Its weight
# gradient walks an expert's slots 64 at a time with the last step from a zero-padded side buffer: fills of exactly
# 0, 64, 128, ... and one past them are the corner cases.  A zero gate matrix with a fixed bias sends every token to the
# same two experts (in bias order), so the fills are T, T, 0, 0.
@pytest.mark.parametrize("T", [1, 63, 64, 65, 128, 129, 192, 256, 257])
def test_layer_train_step_fills_at_reduction_step_boundaries(moe, T):
    cfg = synth.CONFIGS[1].scaled(T=T, M=256, H=512, E=4, k=2, f=2.0)
    inp = synth.make_inputs(cfg, seed=31, bias_std=0.25)
    inp["Wg"] = np.zeros_like(inp["Wg"])
    inp["gate_bias"] = np.array([0.5, -1.0, 1.5, -2.0], dtype=np.float32)
    d_out = synth.make_inputs(cfg.scaled(cfg_id=53), seed=32)["x"]
    ref = O.moe_layer_backward(inp["x"], inp["Wg"], inp["gate_bias"], inp["W1"], inp["b1"], inp["W2"], inp["b2"],
                               cfg.k, cfg.f, cfg.normalize, cfg.act, d_out)
    assert ref["forward"]["counts"].tolist() == [T, 0, T, 0]
    d = cfg.dtype
    tl = moe.TrainLayer(dev(inp["Wg"], d), torch.from_numpy(inp["gate_bias"]).cuda(), dev(inp["W1"], d), dev(inp["b1"], d),
                        dev(inp["W2"], d), dev(inp["b2"], d), T=cfg.T, k=cfg.k, f=cfg.f, normalize=cfg.normalize, act=cfg.act)
    xd, dod = dev(inp["x"], d), dev(d_out, d)
    out = tl.forward(xd)
    g = tl.backward(xd, dod)
    torch.cuda.synchronize()
    assert_close(host(out), ref["forward"]["out"], d, "out")
    for name in ("dx", "dW1", "db1", "dW2", "db2"):
        assert_close(host(g[name]), ref[name], d, name)
    for e in (1, 3):                                                # experts without a token: exactly zero gradients
        assert (host(g["dW1"])[e].view(np.uint32) << 1 == 0).all() and (host(g["dW2"])[e].view(np.uint32) << 1 == 0).all()


# ----------------------------------------------------------------------------------------------------------------
# the layer call allocates nothing, clears nothing by memset and never synchronises: it can be captured in a HIP graph
# ----------------------------------------------------------------------------------------------------------------
def test_layer_forward_in_hip_graph(moe):
    cfg = synth.CONFIGS[1].scaled(T=1500, M=256, H=512, E=8)
    inp = synth.make_inputs(cfg, seed=21, bias_std=0.25)
    d = cfg.dtype
    layer = moe.MoELayer(dev(inp["Wg"], d), None, dev(inp["W1"], d), dev(inp["b1"], d), dev(inp["W2"], d), dev(inp["b2"], d),
                         T=cfg.T, k=cfg.k, f=cfg.f, normalize=cfg.normalize, act=cfg.act)
    x = dev(inp["x"], d)
    eager = layer.forward(x).clone()
    torch.cuda.synchronize()
    static_x = x.clone()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        static_out = layer.forward(static_x)
    other = dev(synth.make_inputs(cfg, seed=22)["x"], d)
    eager_other = layer.forward(other).clone()
    for rep in range(3):                                            # replays with eager work and synchronisation in between
        static_x.copy_(x if rep != 1 else other)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(static_out, eager if rep != 1 else eager_other), rep
        layer.forward(other)
        torch.cuda.synchronize()


# ----------------------------------------------------------------------------------------------------------------
# dispatch fused into the first expert GEMM: same results as encode + FFN on the rows that exist
# ----------------------------------------------------------------------------------------------------------------
FUSED_LAYERS = [
    synth.CONFIGS[1].scaled(T=1500, M=256, H=512, E=8),
    synth.CONFIGS[2].scaled(T=1960, M=768, H=1024, E=32),
    synth.CONFIGS[3].scaled(T=4096, M=256, H=512, E=64),
    synth.CONFIGS[4].scaled(T=4096, M=512, H=256, E=128),
    synth.CONFIGS[1].scaled(T=2000, M=264, H=520, E=8),                   # unsupported by the fused kernel: falls back
]


@pytest.mark.parametrize("cfg", FUSED_LAYERS, ids=lambda c: f"{c.name}-T{c.T}-M{c.M}-H{c.H}-E{c.E}")
def test_layer_fused_dispatch(moe, cfg):
    inp = synth.make_inputs(cfg, seed=5, bias_std=0.25)
    ref = O.moe_layer(inp["x"], inp["Wg"], inp["gate_bias"], inp["W1"], inp["b1"], inp["W2"], inp["b2"],
                      cfg.k, cfg.f, cfg.normalize, cfg.act, tier="sparse")
    d = cfg.dtype
    layer = moe.MoELayer(dev(inp["Wg"], d), None if inp["gate_bias"] is None else torch.from_numpy(inp["gate_bias"]).cuda(),
                         dev(inp["W1"], d), dev(inp["b1"], d), dev(inp["W2"], d), dev(inp["b2"], d),
                         T=cfg.T, k=cfg.k, f=cfg.f, normalize=cfg.normalize, act=cfg.act, keep_routing=True)
    xd = dev(inp["x"], d)
    plain = host(layer.forward(xd)).copy()
    fused = host(layer.forward(xd, fuse_dispatch=True)).copy()
    torch.cuda.synchronize()
    assert_routing_equal(layer.routing, ref, ref["C"], cfg.name)
    assert_close(fused, ref["out"], cfg.dtype, f"fused-dispatch layer output ({cfg.name})")
    assert np.array_equal(fused.view(np.uint32), plain.view(np.uint32))       # same arithmetic on the same rows


def test_expert_ffn_gather_matches_two_calls(moe):
    cfg = synth.CONFIGS[1].scaled(T=1200, M=128, H=256, E=6)
    inp = synth.make_inputs(cfg, seed=9, bias_std=0.25)
    d = cfg.dtype
    C = O.capacity(cfg.T, cfg.E, cfg.k, cfg.f)
    logits = torch.from_numpy(O.gate_logits(inp["x"], inp["Wg"], inp["gate_bias"])).cuda()
    r = moe.gate_topk(logits, cfg.k, C, cfg.normalize)
    xd, W1, b1, W2, b2 = dev(inp["x"], d), dev(inp["W1"], d), dev(inp["b1"], d), dev(inp["W2"], d), dev(inp["b2"], d)
    Y2 = moe.expert_ffn(moe.encode(xd, r["idx"], r["loc"], r["slot_src"], cfg.E, C), W1, b1, W2, b2, cfg.act, counts=r["counts"])
    Y1 = moe.expert_ffn_gather(xd, r["slot_src"], W1, b1, W2, b2, cfg.act, counts=r["counts"])
    torch.cuda.synchronize()
    filled = (r["slot_src"] >= 0).cpu().numpy()
    assert filled.sum() == int(np.minimum(r["counts"].cpu().numpy(), C).sum())
    assert np.array_equal(host(Y1)[filled].view(np.uint32), host(Y2)[filled].view(np.uint32))


# ----------------------------------------------------------------------------------------------------------------
# dynamic capacity factor (capacity_setting 0, negative, positive): capacity chosen on the device from the arrivals
# ----------------------------------------------------------------------------------------------------------------
DYNAMIC_LAYERS = [
    synth.CONFIGS[0].scaled(T=300, M=40, H=72, E=3),
    synth.CONFIGS[1].scaled(T=1500, M=256, H=512, E=8),
    synth.CONFIGS[3].scaled(T=4096, M=256, H=512, E=64),                  # Zipf-skewed gate: far from balanced arrivals
]


def oracle_dynamic_layer(inp, cfg, setting, C_max=None, bpr=False, cosine=None):
    """The dynamic-capacity layer composed from the oracle's pinned pieces: logits (linear or cosine) -> arrivals ->
    capacity (Sec. 4.1; never above C_max) -> routing at that capacity -> dispatch -> experts -> combine."""
    T, E, k = cfg.T, cfg.E, cfg.k
    if cosine is None:
        logits = O.gate_logits(inp["x"], inp["Wg"], inp["gate_bias"])
    else:
        logits = O.cosine_gate_logits(inp["x"], cosine["Wp"], cosine["Me"], cosine["tau"])
    arrivals = O.route(logits, k, 1, cfg.normalize, bpr=bpr)["counts"]
    C = O.dynamic_capacity(arrivals, T, E, k, setting)
    if C_max is not None:
        C = min(C, C_max)
    r = O.route(logits, k, C, cfg.normalize, bpr=bpr)
    Z = O.encode_sparse(inp["x"], r["idx"], r["loc"], E, C)
    Y = O.expert_ffn(Z, inp["W1"], inp["b1"], inp["W2"], inp["b2"], cfg.act, rows=r["counts"])
    r.update(C=C, logits=logits, out=O.decode_sparse(Y, r["idx"], r["loc"], r["gate_w"], C))
    return r


def run_dynamic(moe, cfg, inp, setting, **kw):
    d = cfg.dtype
    gb = None if inp["gate_bias"] is None else torch.from_numpy(inp["gate_bias"]).cuda()
    got = moe.layer_forward_dynamic(dev(inp["x"], d), dev(inp["Wg"], d), gb, dev(inp["W1"], d), dev(inp["b1"], d),
                                    dev(inp["W2"], d), dev(inp["b2"], d), cfg.k, setting, cfg.normalize, cfg.act, **kw)
    torch.cuda.synchronize()
    return got


@pytest.mark.parametrize("cfg", DYNAMIC_LAYERS, ids=lambda c: f"{c.name}-T{c.T}-E{c.E}")
@pytest.mark.parametrize("setting", [0.0, -0.5, -1.0, -64.0, 1.25])
def test_layer_dynamic_capacity(moe, cfg, setting):
    """moe_layer_forward_dynamic (one C call, capacity chosen and used on the device) against the oracle's layer with
    the same capacity setting; buffers sized for C_max = T."""
    inp = synth.make_inputs(cfg, seed=3, bias_std=0.25)
    ref = O.moe_layer(inp["x"], inp["Wg"], inp["gate_bias"], inp["W1"], inp["b1"], inp["W2"], inp["b2"],
                      cfg.k, cfg.f, cfg.normalize, cfg.act, tier="sparse", capacity_setting=setting)
    got = run_dynamic(moe, cfg, inp, setting)
    assert got["C"] == ref["C"]
    assert got["needed_capacity"] == int(ref["counts"].max())
    if setting == 0:
        assert ref["kept"].all()
    assert_routing_equal(got, ref, ref["C"], cfg.name)
    assert_close(host(got["out"]), ref["out"], cfg.dtype, f"dynamic-capacity layer output ({cfg.name}, setting {setting})")
    dead = (~ref["kept"]).all(axis=1)
    assert (host(got["out"])[dead].view(np.uint32) == 0).all()


@pytest.mark.parametrize("cfg", DYNAMIC_LAYERS[1:], ids=lambda c: f"{c.name}-T{c.T}-E{c.E}")
def test_layer_dynamic_capacity_bounded_buffers(moe, cfg):
    """Buffers sized below the needed capacity: setting 0 then behaves like the negative setting with that bound; a
    static factor that does not fit is refused."""
    inp = synth.make_inputs(cfg, seed=4, bias_std=0.25)
    C_max = O.capacity(cfg.T, cfg.E, cfg.k, 0.5)
    ref = oracle_dynamic_layer(inp, cfg, 0.0, C_max=C_max)
    assert ref["C"] == C_max and not ref["kept"].all()                         # the bound really cuts
    same = O.moe_layer(inp["x"], inp["Wg"], inp["gate_bias"], inp["W1"], inp["b1"], inp["W2"], inp["b2"], cfg.k, cfg.f,
                       cfg.normalize, cfg.act, tier="sparse", capacity_setting=-0.5)
    assert same["C"] == C_max and np.array_equal(same["out"], ref["out"])
    got = run_dynamic(moe, cfg, inp, 0.0, C_max=C_max)
    assert got["C"] == C_max and got["needed_capacity"] == int(ref["counts"].max())
    assert_routing_equal(got, ref, C_max, cfg.name)
    assert_close(host(got["out"]), ref["out"], cfg.dtype, "bounded buffers")
    with pytest.raises(moe.MoEError) as err:
        run_dynamic(moe, cfg, inp, 1.0, C_max=C_max)
    assert err.value.status == moe.INVALID_ARG


@pytest.mark.parametrize("cfg", DYNAMIC_LAYERS[1:], ids=lambda c: f"{c.name}-T{c.T}-E{c.E}")
@pytest.mark.parametrize("setting", [0.0, -0.75, 1.0])
def test_layer_dynamic_batch_prioritized(moe, cfg, setting):
    inp = synth.make_inputs(cfg, seed=6, bias_std=0.25)
    ref = oracle_dynamic_layer(inp, cfg, setting, bpr=True)
    got = run_dynamic(moe, cfg, inp, setting, bpr=True)
    assert got["C"] == ref["C"]
    assert_routing_equal(got, ref, ref["C"], f"{cfg.name} BPR")
    assert_close(host(got["out"]), ref["out"], cfg.dtype, f"dynamic-capacity layer, batch prioritized routing, setting {setting}")
    if setting < 0:                                                            # the order matters: token order drops other tokens
        plain = oracle_dynamic_layer(inp, cfg, setting, bpr=False)
        assert not np.array_equal(plain["kept"], ref["kept"])


@pytest.mark.parametrize("cfg", DYNAMIC_LAYERS[1:], ids=lambda c: f"{c.name}-T{c.T}-E{c.E}")
@pytest.mark.parametrize("setting,bpr", [(0.0, False), (-1.0, True), (1.25, False)])
def test_layer_dynamic_cosine_router(moe, cfg, setting, bpr):
    inp = synth.make_inputs(cfg, seed=7, bias_std=0.25)
    rng = np.random.default_rng(cfg.T)
    D = 64
    Wp = synth.round_to_bf16((rng.standard_normal((cfg.M, D)) / np.sqrt(cfg.M)).astype(np.float32))
    Me = rng.standard_normal((cfg.E, D)).astype(np.float32)
    cos = dict(Wp=Wp, Me=Me, tau=0.07)
    ref = oracle_dynamic_layer(inp, cfg, setting, bpr=bpr, cosine=cos)
    inp2 = dict(inp, Wg=Wp, gate_bias=None)
    got = run_dynamic(moe, cfg, inp2, setting, bpr=bpr, cosine_Me=torch.from_numpy(Me).cuda(), cosine_tau=0.07)
    assert got["C"] == ref["C"]
    check_logits(got["logits"].cpu().numpy(), ref["logits"], floor=1.5)
    assert_routing_equal(got, ref, ref["C"], f"{cfg.name} cosine")
    assert_close(host(got["out"]), ref["out"], cfg.dtype, f"dynamic-capacity layer, cosine router, setting {setting}")


def test_layer_dynamic_in_hip_graph(moe):
    """No host synchronisation, allocation or memset inside moe_layer_forward_dynamic: captured once, replayed on
    different inputs (whose arrivals give different capacities), bit-identical to the eager call every time."""
    cfg = synth.CONFIGS[3].scaled(T=4096, M=256, H=512, E=64)
    inp = synth.make_inputs(cfg, seed=21, bias_std=0.25)
    d = cfg.dtype
    layer = moe.DynamicLayer(dev(inp["Wg"], d), torch.from_numpy(inp["gate_bias"]).cuda(), dev(inp["W1"], d), dev(inp["b1"], d),
                             dev(inp["W2"], d), dev(inp["b2"], d), T=cfg.T, k=cfg.k, capacity_setting=0.0,
                             normalize=cfg.normalize, act=cfg.act, C_max=cfg.T)
    xs = [dev(inp["x"], d), dev(synth.make_inputs(cfg, seed=22)["x"], d), dev(synth.make_inputs(cfg, seed=23)["x"][::-1].copy(), d)]
    eager = []
    for x in xs:
        out = layer.forward(x).clone()
        torch.cuda.synchronize()
        eager.append((out, layer.routing["C"].clone(), layer.routing["loc"].clone()))
    assert len({int(c[0]) for _, c, _ in eager}) > 1, "the inputs should need different capacities"
    static_x = xs[0].clone()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        static_out = layer.forward(static_x)
    for rep in (0, 1, 2, 1, 0):                                     # replays with eager work and synchronisation in between
        static_x.copy_(xs[rep])
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(static_out, eager[rep][0]), rep
        assert torch.equal(layer.routing["C"], eager[rep][1]) and torch.equal(layer.routing["loc"], eager[rep][2])
        layer.forward(xs[(rep + 1) % 3])
        torch.cuda.synchronize()


# ----------------------------------------------------------------------------------------------------------------
# moe_layer_forward at the full benchmark sizes, in the launch configuration bench.py times
# ----------------------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("cfg", synth.CONFIGS[1:4], ids=lambda c: c.name)
def test_layer_full_size(moe, cfg):
    print(f"[full-size] {cfg.name}: generating inputs", flush=True)
    inp = synth.make_inputs(cfg, seed=0)
    print("[full-size] oracle", flush=True)
    ref = O.moe_layer(inp["x"], inp["Wg"], inp["gate_bias"], inp["W1"], inp["b1"], inp["W2"], inp["b2"],
                      cfg.k, cfg.f, cfg.normalize, cfg.act, tier="sparse")
    print("[full-size] HIP path", flush=True)
    layer, out = run_layer(moe, cfg, inp)
    check_routed_logits(layer.routing["logits"].cpu().numpy(), ref["logits"])
    assert_routing_equal(layer.routing, ref, ref["C"], cfg.name)
    plain = host(out).copy()
    assert_close(plain, ref["out"], cfg.dtype, f"layer output ({cfg.name})")
    fused = host(layer.forward(dev(inp["x"], cfg.dtype), fuse_dispatch=True))
    assert np.array_equal(fused.view(np.uint32), plain.view(np.uint32)), "fused dispatch must reproduce the plain path bit for bit"


def test_layer_backward_full_size(moe):
    """The benchmark workload's whole training step (moe_layer_forward_train + moe_layer_backward) element by element
    against the oracle's layer backward (about a minute of fp64 numpy)."""
    cfg = synth.CONFIGS[1]
    print("[backward full size] inputs and oracle", flush=True)
    inp = synth.make_inputs(cfg, seed=0, bias_std=0.1)
    d_out = synth.make_inputs(cfg.scaled(cfg_id=52), seed=12)["x"]
    ref = O.moe_layer_backward(inp["x"], inp["Wg"], inp["gate_bias"], inp["W1"], inp["b1"], inp["W2"], inp["b2"],
                               cfg.k, cfg.f, cfg.normalize, cfg.act, d_out)
    print("[backward full size] HIP path", flush=True)
    d = cfg.dtype
    gb = None if inp["gate_bias"] is None else torch.from_numpy(inp["gate_bias"]).cuda()
    tl = moe.TrainLayer(dev(inp["Wg"], d), gb, dev(inp["W1"], d), dev(inp["b1"], d), dev(inp["W2"], d), dev(inp["b2"], d),
                        T=cfg.T, k=cfg.k, f=cfg.f, normalize=cfg.normalize, act=cfg.act)
    xd = dev(inp["x"], d)
    out = tl.forward(xd)
    g = tl.backward(xd, dev(d_out, d))
    torch.cuda.synchronize()
    assert_close(host(out), ref["forward"]["out"], d, "out")
    for name in ("dx", "dWg", "dW1", "db1", "dW2", "db2"):
        assert_close(host(g[name]), ref[name], d, name)
    scale = np.abs(ref["dgate_bias"]).max()
    assert np.abs(g["dgate_bias"].cpu().numpy() - ref["dgate_bias"]).max() <= 2e-2 * max(scale, 1e-30)


def assert_close_on_device(got, ref, dtype, what):
    """assert_close with the comparison arithmetic done in fp64 on the device (the reference comes from the host)."""
    r = torch.from_numpy(np.ascontiguousarray(ref, dtype=np.float64)).cuda()
    g = got.double()
    assert bool(torch.isfinite(g).all()), f"{what}: non-finite values"
    scale = float(r.abs().max())
    err = float((g - r).abs().max())
    assert err <= TOL[dtype] * scale, f"{what}: max abs err {err:.3e} > {TOL[dtype]:.0e} * max|ref| ({scale:.3e})"
    rms = float(((g - r) ** 2).mean().sqrt()) / max(float((r ** 2).mean().sqrt()), 1e-300)
    assert rms <= RMS_TOL[dtype], f"{what}: relative rms err {rms:.3e} > {RMS_TOL[dtype]:.0e}"


def test_layer_full_size_finegrained(moe, progress):
    """T=131072, E=128, top-8, every value: routing in full, then the oracle's expert-by-expert tier evaluates all
    128 slabs (the buffered fp64 oracle would need > 100 GB): every filled row of the dispatch buffer bit for bit and
    every unfilled row +0, every filled row of the expert output and every row of the layer output within tolerance."""
    cfg = synth.CONFIGS[4]
    progress("[finegrained] generating inputs")
    inp = synth.make_inputs(cfg, seed=0)
    C = O.capacity(cfg.T, cfg.E, cfg.k, cfg.f)
    progress("[finegrained] oracle routing")
    logits = O.gate_logits(inp["x"], inp["Wg"], inp["gate_bias"])
    ref = O.route(logits, cfg.k, C, cfg.normalize)
    progress("[finegrained] HIP path")
    d = cfg.dtype
    xd, W1d, W2d = dev(inp["x"], d), dev(inp["W1"], d), dev(inp["W2"], d)
    layer = moe.MoELayer(dev(inp["Wg"], d), None, W1d, None, W2d, None, T=cfg.T, k=cfg.k, f=cfg.f,
                         normalize=cfg.normalize, act=cfg.act, keep_routing=True)
    out = layer.forward(xd).clone()
    fused = layer.forward(xd, fuse_dispatch=True)
    torch.cuda.synchronize()
    assert torch.equal(fused, out), "fused dispatch must reproduce the plain path bit for bit"
    check_routed_logits(layer.routing["logits"].cpu().numpy(), logits)
    assert_routing_equal(layer.routing, ref, C, cfg.name)
    g = layer.routing
    del layer, fused
    torch.cuda.empty_cache()
    # the stage entry points on the same routing: the whole dispatch buffer and the whole expert output
    src = O.slot_source(ref["idx"], ref["loc"], cfg.E, C)
    slot_src = torch.from_numpy(src).cuda()
    Z = moe.encode(xd, g["idx"], g["loc"], slot_src, cfg.E, C)
    Y = moe.expert_ffn(Z, W1d, None, W2d, None, cfg.act, g["counts"])
    torch.cuda.synchronize()
    fills = np.minimum(ref["counts"], C)
    seen = []

    def check_slab(e, tokens, w, Ze, Ye):
        n = len(tokens)
        assert n == fills[e] and np.array_equal(tokens, src[e, :n])
        want_z = torch.from_numpy(synth.bf16_bits(Ze.astype(np.float32)).view(np.int16)).cuda()
        assert torch.equal(Z[e, :n].view(torch.int16), want_z), f"dispatch buffer of expert {e}"
        assert int(Z[e, n:].view(torch.int16).ne(0).sum()) == 0, f"unfilled slots of expert {e} must be +0"
        if n:
            assert_close_on_device(Y[e, :n], Ye, d, f"expert output, expert {e} ({n} rows)")
        seen.append(e)
        if e % 16 == 15:
            progress(f"[finegrained] oracle: {e + 1} of {cfg.E} experts checked")

    want = O.moe_layer_streamed(inp["x"], inp["Wg"], inp["gate_bias"], inp["W1"], None, inp["W2"], None, cfg.k, cfg.f,
                                cfg.normalize, cfg.act, logits=logits, on_expert=check_slab)
    assert seen == list(range(cfg.E))
    del Z, Y
    torch.cuda.empty_cache()
    progress("[finegrained] layer output, all tokens")
    assert_close_on_device(out, want["out"], d, "layer output (all tokens)")
    step = 16384                                                     # and block by block, each against its own scale
    for t0 in range(0, cfg.T, step):
        assert_close_on_device(out[t0:t0 + step], want["out"][t0:t0 + step], d, f"layer output, tokens {t0}..{t0 + step - 1}")
    dead = (~ref["kept"]).all(axis=1)
    assert int(out[torch.from_numpy(dead).cuda()].view(torch.int16).ne(0).sum()) == 0
    del want, out
    # the training step at this size: the parameter gradients of two experts against the oracle's backward of those
    # experts on their own slabs (dY of a slot = gate weight x d_out of its token; Appendix B)
    torch.cuda.empty_cache()
    progress("[finegrained] training step")
    tl = moe.TrainLayer(dev(inp["Wg"], d), None, W1d, None, W2d, None, T=cfg.T, k=cfg.k, f=cfg.f,
                        normalize=cfg.normalize, act=cfg.act)
    d_out = synth.make_inputs(cfg.scaled(cfg_id=52), seed=12)["x"]
    tl.forward(xd)
    grads = tl.backward(xd, dev(d_out, d))
    torch.cuda.synchronize()
    for e in (int(np.argmax(fills)), int(np.argmin(np.where(fills > 0, fills, C + 1)))):
        n = int(fills[e])
        toks = src[e, :n]
        w = np.zeros(n)
        for j in range(cfg.k):
            hit = (ref["idx"][toks, j] == e) & (ref["loc"][toks, j] == np.arange(n))
            w[hit] = ref["gate_w"][toks[hit], j]
        want_g = O.ffn_rows_backward(inp["x"][toks], inp["W1"][e], None, inp["W2"][e], w[:, None] * d_out[toks].astype(np.float64), cfg.act)
        for name in ("dW1", "db1", "dW2", "db2"):
            assert_close(host(grads[name][e]), want_g[name], d, f"{name} of expert {e} ({n} slots)")
