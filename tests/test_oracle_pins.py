"""Pins of the CPU oracle against things other than itself (CPU only).

Each check takes the oracle module as an argument so that `test_planted_mistakes_are_caught` can run the same
checks on copies of the oracle with one deliberate mistake each and see them fail.
"""
import itertools
import math
import os
import types

import numpy as np
import pytest
import torch

from oracle import moe_oracle as ORACLE

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLDEN = os.path.join(ROOT, "tests", "golden")


def _rng(seed):
    return np.random.default_rng(seed)


def _tiny_layer_inputs(seed, T, M, H, E, bias=True):
    r = _rng(seed)
    x = r.standard_normal((T, M)).astype(np.float32)
    Wg = (r.standard_normal((M, E)) / math.sqrt(M)).astype(np.float32)
    gb = r.standard_normal(E).astype(np.float32) * 0.1 if bias else None
    W1 = (r.standard_normal((E, M, H)) / math.sqrt(M)).astype(np.float32)
    W2 = (r.standard_normal((E, H, M)) / math.sqrt(H)).astype(np.float32)
    b1 = r.standard_normal((E, H)).astype(np.float32) * 0.1 if bias else None
    b2 = r.standard_normal((E, M)).astype(np.float32) * 0.1 if bias else None
    return x, Wg, gb, W1, b1, W2, b2


def _torch_act(h, act):
    if act == ORACLE.ACT_RELU:
        return torch.relu(h)
    if act == ORACLE.ACT_GELU:
        return torch.nn.functional.gelu(h, approximate="none")
    return torch.nn.functional.silu(h)


# ----------------------------------------------------------------------------------------------------------------
# individual pins (o = oracle module under test)
# ----------------------------------------------------------------------------------------------------------------

def pin_capacity_golden(o):
    for line in open(os.path.join(GOLDEN, "capacity_eq1.txt")):
        line = line.split("#")[0].strip()
        if not line:
            continue
        T, E, k, f, C = line.split()
        assert o.capacity(int(T), int(E), int(k), float(f)) == int(C), line


def _read_worked_example():
    blocks, name = {}, None
    for line in open(os.path.join(GOLDEN, "routing_worked_example.txt")):
        line = line.split("#")[0].rstrip()
        if not line.strip():
            continue
        if line.strip().isalpha():
            name = line.strip()
            blocks[name] = []
        else:
            blocks[name].append([float(v) for v in line.split()])
    return {k: np.array(v) for k, v in blocks.items()}


def pin_worked_routing_example(o):
    g = _read_worked_example()
    logits = g["logits"].astype(np.float32)
    T, E = logits.shape
    C = o.capacity(T, E, 2, 1.0)
    assert C == 4
    r = o.route(logits, 2, C, 1)
    assert np.array_equal(r["idx"], g["idx"].astype(np.int32))
    assert np.array_equal(r["loc"], g["loc"].astype(np.int32))
    assert np.array_equal(r["kept"], g["kept"].astype(bool))
    assert np.array_equal(r["counts"], g["counts"].astype(np.int32).ravel())
    # gate weights of token 0: softmax(3,1,2) -> p0, p2 renormalised over the two choices
    e = np.exp(np.array([3.0, 1.0, 2.0]) - 3.0)
    p = e / e.sum()
    np.testing.assert_allclose(r["gate_w"][0], [p[0] / (p[0] + p[2]), p[2] / (p[0] + p[2])], rtol=1e-14)


def pin_fig2_even_top1(o):
    """Fig. 2: 2 samples x 6 tokens, 3 experts, evenly dispatched top-1, f = 1 -> C = 4, every slot filled once."""
    T, E, M = 12, 3, 5
    C = o.capacity(T, E, 1, 1.0)
    assert C == 4
    pref = np.array([0, 1, 2, 2, 0, 1, 1, 2, 0, 0, 1, 2])     # four tokens per expert
    logits = np.full((T, E), -1.0, dtype=np.float32)
    logits[np.arange(T), pref] = 1.0
    r = o.route(logits, 1, C, 0)
    assert r["kept"].all() and np.array_equal(r["counts"], [4, 4, 4])
    x = _rng(1).standard_normal((T, M)).astype(np.float32)
    D, W = o.dense_masks(r["idx"], r["loc"], r["gate_w"], E, C)
    assert D.sum() == 12 and (D.sum(axis=0) == 1).all() and (D.sum(axis=(1, 2)) == 1).all()
    Z = o.encode_dense(D, x).reshape(E * C, M)
    src = o.slot_source(r["idx"], r["loc"], E, C).ravel()
    assert sorted(src.tolist()) == list(range(T))          # Z is a row permutation of x
    assert np.array_equal(Z, x[src].astype(np.float64))
    # expert e holds its tokens in token order
    for e in range(E):
        assert np.array_equal(src.reshape(E, C)[e], np.nonzero(pref == e)[0])


def pin_exhaustive_top1_locations(o):
    """All E^T top-1 routings for small T, E: cumsum-based locations == sequential arrival simulation."""
    for T, E in ((4, 2), (5, 3), (6, 3)):
        for C in (1, 2, T):
            for assign in itertools.product(range(E), repeat=T):
                idx = np.array(assign, dtype=np.int32)[:, None]
                loc, counts = o.slot_locations(idx, E)
                seen = [0] * E
                for t, e in enumerate(assign):
                    assert loc[t, 0] == seen[e]
                    seen[e] += 1
                assert counts.tolist() == seen


def pin_random_topk_vs_bruteforce(o):
    for seed, (T, E, k) in enumerate([(17, 4, 2), (33, 8, 3), (64, 5, 5), (40, 8, 1), (29, 6, 4)]):
        r = _rng(100 + seed)
        logits = (np.round(r.standard_normal((T, E)) * 2) / 2).astype(np.float32)   # coarse grid -> many exact ties
        for f in (0.5, 1.0, 2.0):
            C = o.capacity(T, E, k, f)
            got = o.route(logits, k, C, 1)
            idx, loc, kept, counts = o.brute_force_route(logits, k, C)
            assert np.array_equal(got["idx"], idx)
            assert np.array_equal(got["loc"], loc)
            assert np.array_equal(got["kept"], kept)
            assert np.array_equal(got["counts"], counts)


def pin_invariants(o):
    T, E, k = 600, 16, 3
    logits = (np.round(_rng(7).standard_normal((T, E)) * 4) / 4).astype(np.float32)
    logits[:, 0] += 1.0                                   # skew so that expert 0 overflows
    C = o.capacity(T, E, k, 1.0)
    r = o.route(logits, k, C, 1)
    idx, loc, kept, counts = r["idx"], r["loc"], r["kept"], r["counts"]
    assert all(len(set(row)) == k for row in idx.tolist())                     # k distinct experts per token
    assert counts.sum() == T * k and counts.max() > C                          # something is dropped
    for e in range(E):
        sel = idx == e
        assert sel.sum() == counts[e]
        assert sorted(loc[sel].tolist()) == list(range(counts[e]))            # arrival positions are a bijection
        assert (kept & sel).sum() == min(counts[e], C)
        assert sorted(loc[sel & kept].tolist()) == list(range(min(counts[e], C)))
        for j in range(k - 1):                                                 # rank j entirely before rank j+1
            a, b = loc[sel[:, j], j], loc[sel[:, j + 1], j + 1]
            if a.size and b.size:
                assert a.max() < b.min()
        for j in range(k):                                                     # token order within a rank
            assert (np.diff(loc[sel[:, j], j]) > 0).all()
    # selected logits are the k largest, in non-increasing order
    srt = -np.sort(-logits, axis=1)[:, :k]
    assert np.array_equal(logits[np.arange(T)[:, None], idx], srt)
    np.testing.assert_allclose(r["gate_w"].sum(axis=1), 1.0, rtol=1e-13)
    # minimum no-drop capacity (Sec. 4.1, dynamic capacity factor = 0) is max_e counts
    r2 = o.route(logits, k, int(counts.max()), 1)
    assert r2["kept"].all()
    r3 = o.route(logits, k, int(counts.max()) - 1, 1)
    assert (~r3["kept"]).sum() == (counts == counts.max()).sum()


def pin_ties_lower_index(o):
    T, E = 9, 6
    eq = np.zeros((T, E), dtype=np.float32)
    assert np.array_equal(o.topk_experts(eq, 4), np.tile(np.arange(4, dtype=np.int32), (T, 1)))
    dup = np.array([[1.0, 5.0, 5.0, 0.0, 5.0, -2.0]], dtype=np.float32)
    assert o.topk_experts(dup, 4).tolist() == [[1, 2, 4, 0]]
    z = np.array([[-0.0, 0.0, -1.0]], dtype=np.float32)
    assert o.topk_experts(z, 2).tolist() == [[0, 1]]
    z = np.array([[0.0, -0.0, -1.0]], dtype=np.float32)
    assert o.topk_experts(z, 2).tolist() == [[0, 1]]


def pin_gate_against_torch(o):
    x, Wg, gb, *_ = _tiny_layer_inputs(3, 50, 24, 8, 7)
    ref = (torch.from_numpy(x).double() @ torch.from_numpy(Wg).double() + torch.from_numpy(gb).double()).float().numpy()
    got = o.gate_logits(x, Wg, gb, rows_per_pass=16)
    assert got.dtype == np.float32
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-6)
    assert (got != ref).mean() < 0.05                    # identical up to the odd last-bit rounding of the fp64 sum
    p = o.softmax_rows(got)
    np.testing.assert_allclose(p, torch.softmax(torch.from_numpy(got).double(), dim=1).numpy(), rtol=1e-13)
    k = 3
    tv, ti = torch.topk(torch.from_numpy(got), k, dim=1, largest=True, sorted=True)   # tie-free random logits
    assert np.array_equal(o.topk_experts(got, k), ti.numpy().astype(np.int32))
    w = o.gate_weights(p, ti.numpy(), 1)
    tw = torch.gather(torch.from_numpy(p), 1, ti)
    np.testing.assert_allclose(w, (tw / tw.sum(1, keepdim=True)).numpy(), rtol=1e-13)
    w0 = o.gate_weights(p, ti.numpy(), 0)
    np.testing.assert_allclose(w0, tw.numpy(), rtol=1e-15)


def pin_activations_and_ffn_against_torch(o):
    h = np.linspace(-6, 6, 241)
    for act in (o.ACT_RELU, o.ACT_GELU, o.ACT_SILU):
        np.testing.assert_allclose(o.activation(h, act), _torch_act(torch.from_numpy(h), act).numpy(), rtol=1e-12, atol=1e-15)
    # E = 1, k = 1, C >= T: the layer is 1.0 * a dense two-layer MLP
    for act in (o.ACT_RELU, o.ACT_GELU, o.ACT_SILU):
        x, Wg, gb, W1, b1, W2, b2 = _tiny_layer_inputs(5 + act, 21, 12, 20, 1)
        r = o.moe_layer(x, Wg, gb, W1, b1, W2, b2, k=1, f=1.0, normalize=0, act=act, tier="dense")
        tx = torch.from_numpy(x).double()
        ref = torch.nn.functional.linear(
            _torch_act(torch.nn.functional.linear(tx, torch.from_numpy(W1[0]).double().T, torch.from_numpy(b1[0]).double()), act),
            torch.from_numpy(W2[0]).double().T, torch.from_numpy(b2[0]).double())
        np.testing.assert_allclose(r["out"], ref.numpy(), rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(r["gate_w"], 1.0, rtol=1e-15)


def pin_no_drop_equals_weighted_sum_of_experts(o):
    """C >= T (f >= E/k): nothing is dropped, so out[t] = sum_j w[t,j] FFN_{idx[t,j]}(x[t]) -- evaluated with torch."""
    T, M, H, E, k = 37, 16, 24, 4, 2
    x, Wg, gb, W1, b1, W2, b2 = _tiny_layer_inputs(11, T, M, H, E)
    for tier in ("dense", "sparse"):
        r = o.moe_layer(x, Wg, gb, W1, b1, W2, b2, k=k, f=float(E) / k, normalize=1, act=o.ACT_GELU, tier=tier)
        assert r["C"] == T and r["kept"].all()
        tl = torch.from_numpy(r["logits"]).double()
        tp = torch.softmax(tl, dim=1)
        tv, ti = torch.topk(tl, k, dim=1)
        tw = torch.gather(tp, 1, ti)
        tw = tw / tw.sum(1, keepdim=True)
        tx = torch.from_numpy(x).double()
        ref = torch.zeros(T, M, dtype=torch.float64)
        for e in range(E):
            y = _torch_act(tx @ torch.from_numpy(W1[e]).double() + torch.from_numpy(b1[e]).double(), o.ACT_GELU)
            y = y @ torch.from_numpy(W2[e]).double() + torch.from_numpy(b2[e]).double()
            for j in range(k):
                m = (ti[:, j] == e).double()[:, None]
                ref += m * tw[:, j:j + 1] * y
        np.testing.assert_allclose(r["out"], ref.numpy(), rtol=1e-11, atol=1e-12)


def pin_identity_experts_masked_scaling(o):
    """W1 = W2 = I, ReLU, x >= 0: decode(encode(x)) scales each row by the sum of its kept gate weights."""
    T, M, E, k = 40, 8, 4, 2
    r_ = _rng(13)
    x = np.abs(r_.standard_normal((T, M))).astype(np.float32)
    Wg = r_.standard_normal((M, E)).astype(np.float32)
    W = np.tile(np.eye(M, dtype=np.float32), (E, 1, 1))
    for tier in ("dense", "sparse"):
        r = o.moe_layer(x, Wg, None, W, None, W, None, k=k, f=0.5, normalize=1, act=o.ACT_RELU, tier=tier)
        assert (~r["kept"]).any() and (~r["kept"]).all(axis=1).any()       # some tokens lose everything
        scale = (r["gate_w"] * r["kept"]).sum(axis=1)
        np.testing.assert_allclose(r["out"], scale[:, None] * x.astype(np.float64), rtol=1e-13, atol=0)
        dead = (~r["kept"]).all(axis=1)
        assert (r["out"][dead] == 0.0).all() and not np.signbit(r["out"][dead]).any()


def pin_dense_equals_sparse_and_direct(o):
    T, M, H, E, k = 48, 12, 20, 6, 3
    x, Wg, gb, W1, b1, W2, b2 = _tiny_layer_inputs(17, T, M, H, E)
    for f in (0.5, 1.0, 1.5):
        d = o.moe_layer(x, Wg, gb, W1, b1, W2, b2, k=k, f=f, normalize=1, act=o.ACT_SILU, tier="dense")
        s = o.moe_layer(x, Wg, gb, W1, b1, W2, b2, k=k, f=f, normalize=1, act=o.ACT_SILU, tier="sparse")
        assert np.array_equal(d["Z"], s["Z"])                        # at most one non-zero term per slot: exact
        np.testing.assert_allclose(d["out"], s["out"], rtol=1e-12, atol=1e-13)
        filled = o.slot_source(d["idx"], d["loc"], E, d["C"]) >= 0
        np.testing.assert_allclose(d["Y"][filled], s["Y"][filled], rtol=1e-12, atol=1e-13)
        direct = o.token_outputs_direct(np.arange(T), x, d["idx"], d["loc"], d["gate_w"], d["C"], W1, b1, W2, b2, o.ACT_SILU)
        np.testing.assert_allclose(direct, d["out"], rtol=1e-12, atol=1e-13)


def pin_bruteforce_layer(o):
    T, M, H, E = 10, 5, 7, 3
    for k, f, norm, act in ((1, 1.0, 0, o.ACT_RELU), (2, 0.75, 1, o.ACT_GELU), (3, 0.5, 1, o.ACT_SILU), (2, 1.0, 0, o.ACT_GELU)):
        x, Wg, gb, W1, b1, W2, b2 = _tiny_layer_inputs(23 + k, T, M, H, E)
        ref = o.brute_force_layer(x, Wg, gb, W1, b1, W2, b2, k, f, norm, act)
        for tier in ("dense", "sparse"):
            r = o.moe_layer(x, Wg, gb, W1, b1, W2, b2, k=k, f=f, normalize=norm, act=act, tier=tier)
            np.testing.assert_allclose(r["out"], ref, rtol=1e-11, atol=1e-12)


def pin_streamed_tier(o):
    """The expert-by-expert tier gives the buffered tiers' result: slabs bit for bit, the output bit for bit with one
    term per token (top-1) and to fp64 rounding of a reordered sum of at most k terms otherwise; also against the
    independent per-token brute force."""
    T, M, H, E = 60, 12, 20, 6
    for k, f, norm, act in ((1, 1.0, 0, o.ACT_RELU), (1, 0.5, 0, o.ACT_GELU), (3, 0.5, 1, o.ACT_SILU), (2, 1.5, 1, o.ACT_GELU), (6, 1.0, 1, o.ACT_SILU)):
        x, Wg, gb, W1, b1, W2, b2 = _tiny_layer_inputs(31 + k, T, M, H, E)
        s = o.moe_layer(x, Wg, gb, W1, b1, W2, b2, k=k, f=f, normalize=norm, act=act, tier="sparse")
        C = s["C"]
        src = o.slot_source(s["idx"], s["loc"], E, C)
        seen = []

        def check(e, tokens, w, Ze, Ye):
            n = len(tokens)
            seen.append(e)
            assert n == min(int(s["counts"][e]), C)
            assert np.array_equal(tokens, src[e, :n]) and (src[e, n:] == -1).all()
            assert np.array_equal(Ze, s["Z"][e, :n]) and np.array_equal(Ye, s["Y"][e, :n])
            for c in range(n):                                       # the weight of the choice that owns the slot
                j = [j for j in range(k) if s["idx"][tokens[c], j] == e and s["loc"][tokens[c], j] == c]
                assert len(j) == 1 and w[c] == s["gate_w"][tokens[c], j[0]]

        r = o.moe_layer_streamed(x, Wg, gb, W1, b1, W2, b2, k=k, f=f, normalize=norm, act=act, on_expert=check)
        assert seen == list(range(E)) and r["C"] == C
        for key in ("idx", "loc", "kept", "counts", "logits"):
            assert np.array_equal(r[key], s[key]), key
        if k == 1:
            assert np.array_equal(r["out"], s["out"])
        np.testing.assert_allclose(r["out"], s["out"], rtol=1e-13, atol=1e-14)
        dead = (~s["kept"]).all(axis=1)
        assert (r["out"][dead] == 0).all()
    T, M, H, E = 10, 5, 7, 3
    x, Wg, gb, W1, b1, W2, b2 = _tiny_layer_inputs(29, T, M, H, E)
    ref = o.brute_force_layer(x, Wg, gb, W1, b1, W2, b2, 2, 0.75, 1, o.ACT_GELU)
    r = o.moe_layer_streamed(x, Wg, gb, W1, b1, W2, b2, k=2, f=0.75, normalize=1, act=o.ACT_GELU)
    np.testing.assert_allclose(r["out"], ref, rtol=1e-11, atol=1e-12)


def pin_dynamic_capacity(o):
    """Sec. 4.1, dynamic capacity factor: x > 0 is Eq. 1 with f = x; x = 0 is the smallest capacity that drops no
    token (so one less must drop one); x < 0 is the same, capped by the capacity of factor -x."""
    # the hand-worked example: arrivals per expert are 6, 2, 4 (T = 6, E = 3, top-2)
    assert o.dynamic_capacity(np.array([6, 2, 4]), 6, 3, 2, 0) == 6
    assert o.dynamic_capacity(np.array([6, 2, 4]), 6, 3, 2, -1.0) == 4       # capped by ceil(2 * 1.0 * 6 / 3)
    assert o.dynamic_capacity(np.array([6, 2, 4]), 6, 3, 2, -2.0) == 6       # cap 8 is above what is needed
    assert o.dynamic_capacity(np.array([6, 2, 4]), 6, 3, 2, 1.25) == 5       # positive: Eq. 1 as it stands
    r_ = _rng(29)
    for T, E, k in ((37, 5, 2), (64, 8, 3), (20, 4, 1)):
        logits = r_.standard_normal((T, E)).astype(np.float32) + np.linspace(0, 1.5, E, dtype=np.float32)[None, :]
        counts = o.route(logits, k, 1, 1)["counts"]
        C0 = o.dynamic_capacity(counts, T, E, k, 0)
        assert o.route(logits, k, C0, 1)["kept"].all()                       # nothing dropped ...
        assert not o.route(logits, k, C0 - 1, 1)["kept"].all()               # ... and no smaller capacity does that
        for x in (0.5, 1.0, 4.0):
            assert o.dynamic_capacity(counts, T, E, k, x) == o.capacity(T, E, k, x)
            Cn = o.dynamic_capacity(counts, T, E, k, -x)
            assert Cn == min(C0, o.capacity(T, E, k, x)) and Cn <= o.capacity(T, E, k, x)
            # the kept set under -x is the kept set of the static factor x
            assert np.array_equal(o.route(logits, k, Cn, 1)["kept"], o.route(logits, k, o.capacity(T, E, k, x), 1)["kept"])
    # through the layer: setting 0 reproduces a static factor that is large enough, and drops nothing
    x, Wg, gb, W1, b1, W2, b2 = _tiny_layer_inputs(31, 30, 6, 9, 4)
    d = o.moe_layer(x, Wg, gb, W1, b1, W2, b2, k=2, f=1.0, normalize=1, act=o.ACT_GELU, tier="dense", capacity_setting=0)
    s_ = o.moe_layer(x, Wg, gb, W1, b1, W2, b2, k=2, f=float(4), normalize=1, act=o.ACT_GELU, tier="dense")
    assert d["kept"].all() and d["C"] == int(d["counts"].max()) and d["C"] <= s_["C"]
    np.testing.assert_allclose(d["out"], s_["out"], rtol=1e-12, atol=1e-13)
    capped = o.moe_layer(x, Wg, gb, W1, b1, W2, b2, k=2, f=1.0, normalize=1, act=o.ACT_GELU, tier="dense", capacity_setting=-0.5)
    static = o.moe_layer(x, Wg, gb, W1, b1, W2, b2, k=2, f=0.5, normalize=1, act=o.ACT_GELU, tier="dense")
    assert not capped["kept"].all()
    np.testing.assert_allclose(capped["out"], static["out"], rtol=1e-12, atol=1e-13)


def pin_encode_decode_backward(o):
    """Appendix B, differentiable encode / decode: the backward maps are the adjoints of the (already pinned) forward
    maps, the gate-weight gradient is the derivative of a map that is linear in the gate weight, and all of it agrees
    with torch's autograd through the dense one-hot einsums."""
    T, M, E, k = 26, 7, 4, 2
    r_ = _rng(41)
    logits = (r_.standard_normal((T, E)) + np.array([2.0, 0.5, 0.0, -2.0])[None, :]).astype(np.float32)
    C = 12                                                  # a skewed gate: some drops and some unfilled slots
    rt = o.route(logits, k, C, 1)
    idx, loc, w = rt["idx"], rt["loc"], rt["gate_w"]
    assert (~rt["kept"]).any() and (o.slot_source(idx, loc, E, C) < 0).any()
    D, W = o.dense_masks(idx, loc, w, E, C)
    x, dZ = r_.standard_normal((T, M)), r_.standard_normal((E, C, M))
    Y, d_out = r_.standard_normal((E, C, M)), r_.standard_normal((T, M))
    # adjoint identities against the forward maps
    dx = o.encode_backward_dense(D, dZ)
    np.testing.assert_allclose((dZ * o.encode_dense(D, x)).sum(), (dx * x).sum(), rtol=1e-12)
    dY = o.decode_backward_dense(W, d_out)
    np.testing.assert_allclose((d_out * o.decode_dense(W, Y)).sum(), (dY * Y).sum(), rtol=1e-12)
    # out is linear in the gate weights: <d_out, out(w)> = sum_{t,j} w[t,j] dgate[t,j]
    dg = o.gate_weight_grad(d_out, Y, idx, loc, C)
    np.testing.assert_allclose((d_out * o.decode_dense(W, Y)).sum(), (w * dg).sum(), rtol=1e-12)
    assert (dg[~rt["kept"]] == 0).all()
    # torch autograd through the dense einsums
    Dt, xt = torch.from_numpy(D), torch.from_numpy(x).requires_grad_(True)
    torch.einsum("tec,tm->ecm", Dt, xt).backward(torch.from_numpy(dZ))
    np.testing.assert_allclose(dx, xt.grad.numpy(), rtol=1e-12, atol=1e-13)
    wt, Yt = torch.from_numpy(w).requires_grad_(True), torch.from_numpy(Y).requires_grad_(True)
    Wt = torch.zeros((T, E, C), dtype=torch.float64)
    for j in range(k):
        t = torch.from_numpy(np.nonzero(rt["kept"][:, j])[0])
        Wt = Wt.index_put((t, torch.from_numpy(idx[t.numpy(), j].astype(np.int64)), torch.from_numpy(loc[t.numpy(), j].astype(np.int64))),
                          wt[t, j], accumulate=True)
    torch.einsum("tec,ecm->tm", Wt, Yt).backward(torch.from_numpy(d_out))
    np.testing.assert_allclose(dY, Yt.grad.numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(dg, wt.grad.numpy(), rtol=1e-12, atol=1e-13)
    # zero-skipping forms are the same sums
    np.testing.assert_allclose(o.encode_backward_sparse(dZ, idx, loc, C), dx, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(o.decode_backward_sparse(d_out, idx, loc, w, E, C), dY, rtol=1e-13, atol=1e-14)
    dead = (~rt["kept"]).all(axis=1)
    assert (o.encode_backward_sparse(dZ, idx, loc, C)[dead] == 0).all()


def pin_ffn_backward(o):
    """Backward of the expert layer against torch autograd through an independent forward, and against central
    finite differences of the oracle's own (pinned) forward; rows past the fill contribute nothing."""
    E, C, M, H = 3, 9, 5, 7
    r_ = _rng(53)
    Z, dY = r_.standard_normal((E, C, M)), r_.standard_normal((E, C, M))
    W1, W2 = r_.standard_normal((E, M, H)) / math.sqrt(M), r_.standard_normal((E, H, M)) / math.sqrt(H)
    b1, b2 = r_.standard_normal((E, H)) * 0.3, r_.standard_normal((E, M)) * 0.3
    rows = [9, 4, 0]
    for act in (o.ACT_RELU, o.ACT_GELU, o.ACT_SILU):
        g = o.expert_ffn_backward(Z, W1, b1, W2, dY, act, rows=rows)
        tZ, tW1, tb1, tW2, tb2 = (torch.from_numpy(a.copy()).requires_grad_(True) for a in (Z, W1, b1, W2, b2))
        loss = 0.0
        for e in range(E):
            n = rows[e]
            y = _torch_act(tZ[e, :n] @ tW1[e] + tb1[e], act) @ tW2[e] + tb2[e]
            loss = loss + (y * torch.from_numpy(dY[e, :n])).sum()
        loss.backward()
        for name, t in (("dZ", tZ), ("dW1", tW1), ("db1", tb1), ("dW2", tW2), ("db2", tb2)):
            np.testing.assert_allclose(g[name], t.grad.numpy(), rtol=1e-9, atol=1e-11, err_msg=f"{name} act {act}")
        assert (g["dZ"][1, 4:] == 0).all() and (g["dZ"][2] == 0).all() and (g["dW1"][2] == 0).all()
        if act != o.ACT_RELU:                               # smooth activations: finite differences of the forward
            def loss_of(Zp, W1p):
                Y = o.expert_ffn(Zp, W1p, b1, W2, b2, act, rows=rows)
                return sum((Y[e, :rows[e]] * dY[e, :rows[e]]).sum() for e in range(E))
            eps = 1e-6
            for (e, c, m) in ((0, 2, 1), (1, 3, 4)):
                Zp, Zm = Z.copy(), Z.copy()
                Zp[e, c, m] += eps
                Zm[e, c, m] -= eps
                np.testing.assert_allclose((loss_of(Zp, W1) - loss_of(Zm, W1)) / (2 * eps), g["dZ"][e, c, m], rtol=1e-6, atol=1e-8)
            Wp, Wm = W1.copy(), W1.copy()
            Wp[1, 2, 3] += eps
            Wm[1, 2, 3] -= eps
            np.testing.assert_allclose((loss_of(Z, Wp) - loss_of(Z, Wm)) / (2 * eps), g["dW1"][1, 2, 3], rtol=1e-6, atol=1e-8)


def pin_cosine_router(o):
    """Appendix, cosine router: against torch's cosine_similarity, scale invariance, the bound |cos| <= 1, an expert
    embedding parallel to a projected token scores 1 / tau, and the temperature floor of 0.01."""
    T, M, D, E = 23, 12, 16, 5
    r_ = _rng(61)
    x = r_.standard_normal((T, M)).astype(np.float32)
    Wp = (r_.standard_normal((M, D)) / math.sqrt(M)).astype(np.float32)
    Me = r_.standard_normal((E, D)).astype(np.float32)
    for tau in (0.07, 1.0):
        got = o.cosine_gate_logits(x, Wp, Me, tau)
        assert got.dtype == np.float32
        proj = torch.from_numpy((x.astype(np.float64) @ Wp.astype(np.float64)).astype(np.float32).astype(np.float64))
        ref = torch.nn.functional.cosine_similarity(proj[:, None, :], torch.from_numpy(Me.astype(np.float64))[None, :, :], dim=2) / tau
        np.testing.assert_allclose(got, ref.numpy(), rtol=2e-7, atol=1e-7)
        assert (np.abs(got) * tau <= 1.0 + 1e-6).all()
        # scaling the tokens or the expert embeddings by powers of two changes nothing (exactly)
        assert np.array_equal(got, o.cosine_gate_logits(4.0 * x, Wp, 0.5 * Me, tau))
    # an embedding parallel to a token's projection: cosine 1
    proj0 = (x[:1].astype(np.float64) @ Wp.astype(np.float64)).astype(np.float32)
    Me2 = Me.copy()
    Me2[3] = 3.0 * proj0[0]
    np.testing.assert_allclose(o.cosine_gate_logits(x, Wp, Me2, 0.5)[0, 3], 2.0, rtol=1e-6)
    Me2[4] = -proj0[0]
    np.testing.assert_allclose(o.cosine_gate_logits(x, Wp, Me2, 0.5)[0, 4], -2.0, rtol=1e-6)
    # temperatures below 0.01 act as 0.01
    assert np.array_equal(o.cosine_gate_logits(x, Wp, Me, 0.001), o.cosine_gate_logits(x, Wp, Me, 0.01))
    np.testing.assert_allclose(o.cosine_gate_logits(x, Wp, Me, 0.01), 100.0 * o.cosine_gate_logits(x, Wp, Me, 1.0).astype(np.float64), rtol=3e-7, atol=1e-6)


def _read_blocks(path):
    blocks, name = {}, None
    for line in open(path):
        line = line.split("#")[0].strip()
        if not line:
            continue
        if line[0].isalpha():
            name = line
            blocks[name] = []
        else:
            blocks[name].append([float(v) for v in line.split()])
    return {k: np.array(v) for k, v in blocks.items()}


def pin_batch_prioritized_routing(o):
    """BPR: the hand-worked example; sequential simulation in priority order; the order is by decreasing largest
    probability with ties to the lower token; with room for everybody it changes no decision; at an overfull expert the
    dropped first choices are exactly the lowest-priority ones."""
    b = _read_blocks(os.path.join(GOLDEN, "bpr_worked_example.txt"))
    logits = b["logits"].astype(np.float32)
    assert np.array_equal(o.bpr_token_order(logits), b["order"].astype(np.int64).ravel())
    r = o.route(logits, 1, 2, 0, bpr=True)
    assert np.array_equal(r["idx"], b["idx"].astype(np.int32)) and np.array_equal(r["loc"], b["loc"].astype(np.int32))
    assert np.array_equal(r["kept"], b["kept"].astype(bool)) and np.array_equal(r["counts"], b["counts"].astype(np.int32).ravel())
    plain = o.route(logits, 1, 2, 0)
    assert not plain["kept"][4, 0] and plain["kept"][2, 0]            # token order drops the most confident token instead
    r_ = _rng(71)
    for T, E, k, C in ((40, 4, 2, 12), (33, 6, 3, 9), (25, 3, 1, 5)):
        logits = (r_.standard_normal((T, E)) + np.linspace(1.0, 0.0, E)[None, :]).astype(np.float32)
        logits[5] = logits[3]                                         # equal priorities: the lower token goes first
        order = o.bpr_token_order(logits)
        p = torch.softmax(torch.from_numpy(logits.astype(np.float64)), dim=1).max(dim=1).values.numpy().astype(np.float32)
        assert sorted(order.tolist()) == list(range(T))
        assert all(p[order[i]] > p[order[i + 1]] or (p[order[i]] == p[order[i + 1]] and order[i] < order[i + 1]) for i in range(T - 1))
        assert list(order).index(3) + 1 == list(order).index(5)
        r = o.route(logits, k, C, 1, bpr=True)
        bi, bl, bk, bc = o.brute_force_route(logits, k, C, order=order)
        assert np.array_equal(r["idx"], bi) and np.array_equal(r["loc"], bl) and np.array_equal(r["kept"], bk) and np.array_equal(r["counts"], bc)
        big = o.route(logits, k, T * k, 1, bpr=True)
        assert big["kept"].all() and np.array_equal(big["idx"], o.route(logits, k, T * k, 1)["idx"])
        assert np.array_equal(r["counts"], o.route(logits, k, C, 1)["counts"])
        # first choices at one expert: every kept token has priority >= every dropped token
        for e in range(E):
            first = np.nonzero(r["idx"][:, 0] == e)[0]
            kept, dropped = first[r["kept"][first, 0]], first[~r["kept"][first, 0]]
            if len(kept) and len(dropped):
                assert p[kept].min() >= p[dropped].max()


def pin_gate_backward(o):
    """Backward of the gate against torch autograd through softmax -> gather -> renormalise and through the linear layer."""
    T, M, E, k = 19, 6, 5, 3
    r_ = _rng(83)
    x = r_.standard_normal((T, M)).astype(np.float32)
    Wg = r_.standard_normal((M, E)).astype(np.float32)
    bias = r_.standard_normal(E).astype(np.float32)
    logits = o.gate_logits(x, Wg, bias)
    idx = o.topk_experts(logits, k)
    dw = r_.standard_normal((T, k))
    for normalize in (0, 1):
        got = o.gate_backward(logits, idx, dw, normalize)
        lt = torch.from_numpy(logits.astype(np.float64)).requires_grad_(True)
        g = torch.softmax(lt, dim=1).gather(1, torch.from_numpy(idx.astype(np.int64)))
        w = g / g.sum(dim=1, keepdim=True) if normalize else g
        (w * torch.from_numpy(dw)).sum().backward()
        np.testing.assert_allclose(got, lt.grad.numpy(), rtol=1e-10, atol=1e-13)
        np.testing.assert_allclose(got.sum(axis=1), 0.0, atol=1e-13)          # softmax: gradients of a row sum to zero
        np.testing.assert_allclose(o.gate_weights(o.softmax_rows(logits), idx, normalize), w.detach().numpy(), rtol=1e-12)
    dl = r_.standard_normal((T, E))
    xt, Wt, bt = (torch.from_numpy(a.astype(np.float64)).requires_grad_(True) for a in (x, Wg, bias))
    ((xt @ Wt + bt) * torch.from_numpy(dl)).sum().backward()
    gb = o.gate_logits_backward(x, Wg, dl)
    np.testing.assert_allclose(gb["dx"], xt.grad.numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(gb["dWg"], Wt.grad.numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(gb["dbias"], bt.grad.numpy(), rtol=1e-12, atol=1e-13)


def pin_layer_backward(o):
    """The whole layer's backward against torch autograd through a dense one-hot-mask implementation of the layer with
    the routing decisions held fixed."""
    T, M, H, E, k = 22, 6, 9, 4, 2
    x, Wg, gb, W1, b1, W2, b2 = _tiny_layer_inputs(91, T, M, H, E)
    d_out = _rng(92).standard_normal((T, M))
    for f, normalize, act in ((0.6, 1, o.ACT_GELU), (1.5, 0, o.ACT_SILU)):
        got = o.moe_layer_backward(x, Wg, gb, W1, b1, W2, b2, k, f, normalize, act, d_out)
        fw = got["forward"]
        C = fw["C"]
        tx, tWg, tgb, tW1, tb1, tW2, tb2 = (torch.from_numpy(a.astype(np.float64)).requires_grad_(True) for a in (x, Wg, gb, W1, b1, W2, b2))
        lg = tx @ tWg + tgb
        lg = lg + (torch.from_numpy(fw["logits"].astype(np.float64)) - lg).detach()    # the method's one rounding of the logits to fp32
        p = torch.softmax(lg, dim=1)
        idx_t = torch.from_numpy(fw["idx"].astype(np.int64))
        g = p.gather(1, idx_t)
        w = g / g.sum(dim=1, keepdim=True) if normalize else g
        D = torch.zeros((T, E, C), dtype=torch.float64)
        Wm = torch.zeros((T, E, C), dtype=torch.float64)
        for j in range(k):
            t = torch.from_numpy(np.nonzero(fw["kept"][:, j])[0])
            e = idx_t[t, j]
            l = torch.from_numpy(fw["loc"][t.numpy(), j].astype(np.int64))
            D = D.index_put((t, e, l), torch.ones(len(t), dtype=torch.float64), accumulate=True)
            Wm = Wm.index_put((t, e, l), w[t, j], accumulate=True)
        Z = torch.einsum("tec,tm->ecm", D, tx)
        Y = torch.stack([_torch_act(Z[e] @ tW1[e] + tb1[e], act) @ tW2[e] + tb2[e] for e in range(E)])
        out = torch.einsum("tec,ecm->tm", Wm, Y)
        np.testing.assert_allclose(out.detach().numpy(), fw["out"], rtol=1e-10, atol=1e-12)
        (out * torch.from_numpy(d_out)).sum().backward()
        for name, t in (("dx", tx), ("dWg", tWg), ("dgate_bias", tgb), ("dW1", tW1), ("db1", tb1), ("dW2", tW2)):
            np.testing.assert_allclose(got[name], t.grad.numpy(), rtol=1e-8, atol=1e-10, err_msg=name)
        # unfilled slots see b2 in the dense form but are combined with weight 0: db2 counts filled slots only
        filled = (o.slot_source(fw["idx"], fw["loc"], E, C) >= 0)
        np.testing.assert_allclose(got["db2"], tb2.grad.numpy(), rtol=1e-8, atol=1e-10)
        assert filled.sum() == fw["kept"].sum()


PINS = [pin_streamed_tier, pin_layer_backward, pin_gate_backward, pin_batch_prioritized_routing, pin_cosine_router, pin_ffn_backward, pin_encode_decode_backward, pin_dynamic_capacity, pin_capacity_golden, pin_worked_routing_example, pin_fig2_even_top1, pin_exhaustive_top1_locations,
        pin_random_topk_vs_bruteforce, pin_invariants, pin_ties_lower_index, pin_gate_against_torch,
        pin_activations_and_ffn_against_torch, pin_no_drop_equals_weighted_sum_of_experts,
        pin_identity_experts_masked_scaling, pin_dense_equals_sparse_and_direct, pin_bruteforce_layer]


@pytest.mark.parametrize("pin", PINS, ids=lambda p: p.__name__)
def test_pin(pin):
    pin(ORACLE)


# ----------------------------------------------------------------------------------------------------------------
# planted mistakes: each edit of the oracle's source must make at least one pin fail
# ----------------------------------------------------------------------------------------------------------------

MISTAKES = {
    "gate_bwd_normalisation_term_dropped": ("        dg = (dw - (dw * w).sum(axis=1, keepdims=True)) / S", "        dg = dw / S"),
    "gate_bwd_softmax_mean_term_dropped": ("    return p * (dp - (p * dp).sum(axis=1, keepdims=True))", "    return p * dp"),
    "gate_bwd_scatter_overwrites": ("    np.add.at(dp, (np.broadcast_to(rows, idx.shape), idx), dg)", "    dp[np.broadcast_to(rows, idx.shape), idx[:, ::-1]] = dg"),
    "gate_linear_bwd_dx_untransposed": ("dx=dl @ Wd.T,", "dx=dl @ Wd.T[::-1],"),
    "gate_linear_bwd_dbias_mean": ("dbias=dl.sum(axis=0)", "dbias=dl.mean(axis=0)"),
    "bpr_lowest_priority_first": ("    return np.argsort(-key.astype(np.float64), kind=\"stable\")", "    return np.argsort(key.astype(np.float64), kind=\"stable\")"),
    "bpr_priority_is_smallest_probability": ("    key = softmax_rows(logits).max(axis=1).astype(np.float32)", "    key = softmax_rows(logits).min(axis=1).astype(np.float32)"),
    "bpr_priority_is_largest_logit": ("    key = softmax_rows(logits).max(axis=1).astype(np.float32)", "    key = np.asarray(logits, dtype=np.float32).max(axis=1)"),
    "bpr_locations_not_scattered_back": ("        loc[order] = loc_o\n", "        loc[:] = loc_o\n"),
    "bpr_order_ignored": ("    loc, counts = slot_locations(idx, E, bpr_token_order(logits) if bpr else None)", "    loc, counts = slot_locations(idx, E, None)"),
    "cosine_token_norm_dropped": ("    cos = (proj @ Md.T) / (nx[:, None] * ne[None, :])", "    cos = (proj @ Md.T) / ne[None, :]"),
    "cosine_expert_norm_dropped": ("    cos = (proj @ Md.T) / (nx[:, None] * ne[None, :])", "    cos = (proj @ Md.T) / nx[:, None]"),
    "cosine_norm_not_rooted": ("    nx = np.maximum(np.sqrt((proj * proj).sum(axis=1)), 1e-12)", "    nx = np.maximum((proj * proj).sum(axis=1), 1e-12)"),
    "cosine_temperature_multiplies": ("    return (cos / max(float(tau), 0.01)).astype(np.float32)", "    return (cos * max(float(tau), 0.01)).astype(np.float32)"),
    "cosine_temperature_floor_missing": ("    return (cos / max(float(tau), 0.01)).astype(np.float32)", "    return (cos / float(tau)).astype(np.float32)"),
    "cosine_projection_rows_reversed": ("    proj = gate_logits(x, Wp, None, rows_per_pass).astype(np.float64)",
                                        "    proj = gate_logits(x, np.asarray(Wp)[::-1], None, rows_per_pass).astype(np.float64)"),
    "ffn_bwd_gelu_grad_drops_density_term": ("        return 0.5 * (1.0 + _erf(h / math.sqrt(2.0))) + h * np.exp(-0.5 * h * h) / math.sqrt(2.0 * math.pi)",
                                             "        return 0.5 * (1.0 + _erf(h / math.sqrt(2.0)))"),
    "ffn_bwd_silu_grad_sign": ("        return sg * (1.0 + h * (1.0 - sg))", "        return sg * (1.0 - h * (1.0 - sg))"),
    "ffn_bwd_act_grad_at_output": ("    dpre = dh * activation_grad(pre, act)", "    dpre = dh * activation_grad(h, act)"),
    "ffn_bwd_w2_rows_reversed": ("    dh = dy @ W2e.T", "    dh = dy @ W2e.T[::-1]"),
    "ffn_bwd_dw2_from_preactivation": ("dW2=h.T @ dy", "dW2=pre.T @ dy"),
    "ffn_bwd_db1_from_dh": ("db1=dpre.sum(axis=0)", "db1=dh.sum(axis=0)"),
    "ffn_bwd_counts_rows_past_fill": ("        n = C if rows is None else int(min(max(rows[e], 0), C))\n        g = ffn_rows_backward(",
                                      "        n = C\n        g = ffn_rows_backward("),
    "encode_bwd_untransposed": ("    return D.reshape(T, E * C) @ np.asarray(dZ, dtype=np.float64).reshape(E * C, -1)",
                                "    return D.reshape(T, E * C)[:, ::-1] @ np.asarray(dZ, dtype=np.float64).reshape(E * C, -1)"),
    "decode_bwd_unweighted": ("    return (W.reshape(T, E * C).T @ np.asarray(d_out, dtype=np.float64)).reshape(E, C, -1)",
                              "    return ((W != 0).astype(np.float64).reshape(T, E * C).T @ np.asarray(d_out, dtype=np.float64)).reshape(E, C, -1)"),
    "gate_grad_counts_dropped": ("        g[t, j] = (do[t] * np.asarray(Y[idx[t, j], loc[t, j]], dtype=np.float64)).sum(axis=1)",
                                 "        g[:, j] = (do * np.asarray(Y[idx[:, j], np.minimum(loc[:, j], C - 1)], dtype=np.float64)).sum(axis=1)"),
    "gate_grad_weighted_twice": ("        g[t, j] = (do[t] * np.asarray(Y[idx[t, j], loc[t, j]], dtype=np.float64)).sum(axis=1)",
                                 "        g[t, j] = 2.0 * (do[t] * np.asarray(Y[idx[t, j], loc[t, j]], dtype=np.float64)).sum(axis=1)"),
    "sparse_encode_bwd_keeps_dropped": ("        dx[t] += np.asarray(dZ[idx[t, j], loc[t, j]], dtype=np.float64)",
                                        "        dx[:] += np.asarray(dZ[idx[:, j], np.minimum(loc[:, j], C - 1)], dtype=np.float64)"),
    "sparse_decode_bwd_unweighted": ("        dY[idx[t, j], loc[t, j]] = gate_w[t, j][:, None] * np.asarray(d_out[t], dtype=np.float64)",
                                     "        dY[idx[t, j], loc[t, j]] = np.asarray(d_out[t], dtype=np.float64)"),
    "dynamic_capacity_least_full_expert": ("needed = int(np.max(np.asarray(counts)))", "needed = int(np.min(np.asarray(counts)))"),
    "dynamic_capacity_mean_fill": ("needed = int(np.max(np.asarray(counts)))", "needed = int(math.ceil(np.mean(np.asarray(counts))))"),
    "dynamic_capacity_bound_ignored": ("    return min(needed, capacity(T, E, k, -x))", "    return needed"),
    "dynamic_capacity_bound_as_floor": ("    return min(needed, capacity(T, E, k, -x))", "    return max(needed, capacity(T, E, k, -x))"),
    "dynamic_capacity_zero_uses_static": ("    if x == 0:\n        return needed", "    if x == 0:\n        return capacity(T, E, k, 1.0)"),
    "streamed_slots_in_token_order": ("    order = np.lexsort((ll, ee))                      # by expert, then by slot", "    order = np.lexsort((tt, ee))"),
    "streamed_weight_of_first_choice": ("        yield e, tokens, np.asarray(gate_w[tokens, jj[a:b]], dtype=np.float64), Ze, Ye", "        yield e, tokens, np.asarray(gate_w[tokens, 0], dtype=np.float64), Ze, Ye"),
    "streamed_keeps_dropped": ("    tt, jj = np.nonzero(loc < C)                      # kept (token, choice) pairs", "    tt, jj = np.nonzero(loc < C + 1)"),
    "streamed_unweighted_sum": ("        out[tokens] += w[:, None] * Ye                # a token", "        out[tokens] += Ye                # a token"),
    "streamed_overwrites_instead_of_adding": ("        out[tokens] += w[:, None] * Ye                # a token", "        out[tokens] = w[:, None] * Ye                # a token"),
    "capacity_floor": ("int(math.ceil(float(k)", "int(math.floor(float(k)"),
    "capacity_drops_k": ("math.ceil(float(k) * float(f)", "math.ceil(float(f)"),
    "ties_to_higher_index": ("idx[:, j] = np.argmax(work, axis=1)", "idx[:, j] = E - 1 - np.argmax(work[:, ::-1], axis=1)"),
    "topk_picks_smallest": ("idx[:, j] = np.argmax(work, axis=1)", "idx[:, j] = np.argmin(np.where(np.isinf(work), np.inf, work), axis=1)"),
    "chosen_expert_not_masked": ("work[rows, idx[:, j]] = -np.inf", "work[rows, idx[:, j]] -= 1.0"),
    "loc_one_based": ("pos = np.cumsum(mask, axis=0) - 1 + counts[None, :]", "pos = np.cumsum(mask, axis=0) + counts[None, :]"),
    "later_ranks_not_offset": ("pos = np.cumsum(mask, axis=0) - 1 + counts[None, :]", "pos = np.cumsum(mask, axis=0) - 1"),
    "kept_off_by_one": ("kept=(loc < C)", "kept=(loc <= C)"),
    "normalize_ignored": ("    if normalize:\n        w = w / w.sum(axis=1, keepdims=True)", "    if False:\n        pass"),
    "softmax_no_denominator": ("return e / e.sum(axis=1, keepdims=True)", "return e"),
    "gate_bias_dropped": ("acc = acc + bd[None, :]", "acc = acc"),
    "gate_weight_transposed": ("@ Wd\n", "@ Wd[:, ::-1]\n"),
    "encode_scaled_by_gate": ("D[t, idx[t, j], loc[t, j]] += 1.0", "D[t, idx[t, j], loc[t, j]] += gate_w[t, j]"),
    "decode_unweighted": ("W[t, idx[t, j], loc[t, j]] += gate_w[t, j]", "W[t, idx[t, j], loc[t, j]] += 1.0"),
    "sparse_decode_unweighted": ("out[t] += gate_w[t, j][:, None] * Y[", "out[t] += Y["),
    "sparse_encode_keeps_dropped": ("        t = np.nonzero(loc[:, j] < C)[0]\n        Z[idx[t, j], loc[t, j]] = x[t]",
                                    "        t = np.nonzero(loc[:, j] < C + 1)[0]\n        Z[idx[t, j], np.minimum(loc[t, j], C - 1)] = x[t]"),
    "gelu_tanh_form": ("0.5 * h * (1.0 + _erf(h / math.sqrt(2.0)))",
                       "0.5 * h * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (h + 0.044715 * h ** 3)))"),
    "silu_sign": ("h / (1.0 + np.exp(-h))", "h / (1.0 + np.exp(h))"),
    "ffn_activation_dropped": ("    h = activation(h, act)\n    y = h @", "    y = h @"),
    "ffn_activation_before_b1": ("    h = np.asarray(z, dtype=np.float64) @ np.asarray(W1e, dtype=np.float64)\n",
                                 "    h = activation(np.asarray(z, dtype=np.float64) @ np.asarray(W1e, dtype=np.float64), act)\n"
                                 "    act = -1\n"),
    "ffn_w2_transposed_block": ("y = h @ np.asarray(W2e, dtype=np.float64)", "y = h @ np.asarray(W2e, dtype=np.float64)[::-1]"),
    "ffn_b2_dropped": ("        y = y + np.asarray(b2e, dtype=np.float64)[None, :]", "        pass"),
    "direct_ignores_drops": ("sel = np.nonzero(loc[tokens, j] < C)[0]", "sel = np.nonzero(loc[tokens, j] >= 0)[0]"),
}


def _mutated_oracle(old, new):
    path = os.path.join(ROOT, "oracle", "moe_oracle.py")
    src = open(path).read()
    assert src.count(old) >= 1, f"mutation anchor not found: {old!r}"
    mod = types.ModuleType("moe_oracle_mutant")
    mod.__file__ = path
    exec(compile(src.replace(old, new, 1), path, "exec"), mod.__dict__)
    return mod


@pytest.mark.parametrize("name", sorted(MISTAKES))
def test_planted_mistakes_are_caught(name):
    old, new = MISTAKES[name]
    mutant = _mutated_oracle(old, new)
    failed = []
    for pin in PINS:
        try:
            pin(mutant)
        except Exception:            # any failure of a pin counts (assertion, shape or index error)
            failed.append(pin.__name__)
    assert failed, f"planted mistake '{name}' passed every pin"
