"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every declared symbol, and its pure
host functions (capacity, workspace sizes, argument validation) behave as the header says."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "moe_mi355x.h")


@pytest.fixture(scope="module")
def moe():
    from paper_2206_03382_amd import moe as m
    if not os.path.exists(m.LIB_PATH):
        from paper_2206_03382_amd.build import build_library
        build_library(verbose=False)
    m.lib()
    return m


def declared_functions(header=HEADER):
    text = re.sub(r"/\*.*?\*/", "", open(header).read(), flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound(moe):
    names = declared_functions()
    assert {"moe_gate_topk", "moe_encode", "moe_expert_ffn", "moe_decode", "moe_layer_forward"} <= set(names)
    handle = ctypes.CDLL(moe.LIB_PATH)
    for n in names:
        assert hasattr(handle, n), f"{n} is declared in the header but not exported"
    assert sorted(moe.SIGNATURES) == names


def test_probe_library_is_separate(moe):
    """The benchmark's measurement aid lives in a library of its own: the product library exports no probe, and the
    probe library exports what its header declares."""
    from paper_2206_03382_amd import probe
    names = declared_functions(os.path.join(ROOT, "include", "moe_mi355x_probe.h"))
    assert names == ["moe_probe_mfma_sustained"]
    handle = ctypes.CDLL(probe.PROBE_LIB_PATH)
    for n in names:
        assert hasattr(handle, n)
    product = ctypes.CDLL(moe.LIB_PATH)
    assert not any(hasattr(product, n) for n in names + ["moe_mfma_sustained_probe", "moe_expert_ffn_clock_probe"])
    assert handle.moe_probe_mfma_sustained(0, 10, 1, 4096, None, None) == 1          # invalid arguments never launch
    assert handle.moe_probe_mfma_sustained(256, 10, 1, None, None, None) == 1


def test_capacity_follows_eq1(moe, golden_dir):
    for line in open(os.path.join(golden_dir, "capacity_eq1.txt")):
        line = line.split("#")[0].strip()
        if line:
            T, E, k, f, C = line.split()
            assert moe.capacity(int(T), int(E), int(k), float(f)) == int(C), line
    for bad in ((0, 4, 1, 1.0), (8, 0, 1, 1.0), (8, 4, 0, 1.0), (8, 4, 5, 1.0), (8, 4, 1, 0.0), (8, 4, 1, -1.0)):
        assert moe.capacity(*bad) == -1


def test_workspace_sizes(moe):
    assert moe.gate_workspace_bytes(1000, 8, 2) == 2 * 16 * 8 * 4           # k * ceil(T/64) * E * sizeof(int32)
    assert moe.gate_workspace_bytes(1000, 8, 9) == 0                       # k > E
    T, M, H, E, k, C = 16384, 2048, 2048, 8, 2, 5120
    need = moe.layer_workspace_bytes(T, M, H, E, k, C, moe.BF16)
    gate = int(moe.lib().moe_gate_route_workspace_bytes(T, M, E, k, moe.BF16))
    assert moe.gate_workspace_bytes(T, E, k) + E * M * 2 + E * 4 + T * 4 <= gate <= moe.gate_workspace_bytes(T, E, k) + E * M * 2 + E * 4 + T * 4 + 4 * 256
    assert int(moe.lib().moe_gate_route_workspace_bytes(T, M, E, k, moe.F32)) == (moe.gate_workspace_bytes(T, E, k) + 255) // 256 * 256
    payload = T * E * 4 + 3 * T * k * 4 + E * 4 + E * C * 4 + gate + 2 * E * C * M * 2 + E * C * H * 2
    assert payload <= need <= payload + 10 * 256
    assert moe.layer_workspace_bytes(T, M + 4, H, E, k, C, moe.BF16) == 0   # M not a multiple of 8
    assert moe.layer_workspace_bytes(T, M, H, E, k, C, 7) == 0              # unknown dtype


def test_layer_memory_grows_linearly_with_tokens(moe):
    # the setting of the paper's memory table (Sec. 4.2: D = H = 4096, top-2, 2 local experts): no [T, E, C] mask exists,
    # so the layer's workspace is linear in tokens/step where the dense formulation's grows with T^2
    M = H = 4096
    E = k = 2
    sizes = []
    for T in (4096, 8192, 16384, 32768):
        C = moe.capacity(T, E, k, 1.0)
        sizes.append(moe.layer_workspace_bytes(T, M, H, E, k, C, moe.BF16))
        assert T < 16384 or sizes[-1] < T * E * C * 2                      # from 16384 tokens on, less than the dense mask alone
    for a, b in zip(sizes, sizes[1:]):
        assert 1.99 < b / a < 2.01


def test_argument_validation_never_launches(moe):
    L = moe.lib()
    assert L.moe_status_string(moe.OK) == b"ok" and b"workspace" in L.moe_status_string(moe.WORKSPACE_TOO_SMALL)
    fake = 4096                                                               # non-null, 16-byte aligned, never dereferenced
    assert L.moe_gate_topk(None, 8, 4, 1, 2, 0, fake, fake, fake, fake, None, fake, 1 << 20, None) == moe.INVALID_ARG
    assert L.moe_gate_topk(fake, 8, 4, 5, 2, 0, fake, fake, fake, fake, None, fake, 1 << 20, None) == moe.INVALID_ARG   # k > E
    assert L.moe_gate_topk(fake, 8, 1024, 1, 2, 0, fake, fake, fake, fake, None, fake, 1 << 20, None) == moe.UNSUPPORTED
    assert L.moe_gate_topk(fake, 8, 4, 1, 2, 0, fake, fake, fake, fake, None, fake, 1, None) == moe.WORKSPACE_TOO_SMALL
    assert L.moe_gate_logits(fake, fake, None, moe.BF16, 8, 12, 4, fake, None) == moe.UNSUPPORTED                      # M % 8
    assert L.moe_encode(fake, 9, fake, fake, None, 8, 16, 4, 1, 2, fake, None) == moe.INVALID_ARG                      # dtype
    assert L.moe_encode(fake + 2, moe.BF16, fake, fake, None, 8, 16, 4, 1, 2, fake, None) == moe.UNSUPPORTED           # alignment
    assert L.moe_expert_ffn(fake, fake, None, fake, None, 5, moe.BF16, None, 4, 2, 16, 16, fake, fake, None) == moe.INVALID_ARG
    assert L.moe_expert_ffn_train(fake, fake, None, fake, None, 0, moe.BF16, None, 4, 2, 16, 16, None, fake, fake, None) == moe.INVALID_ARG  # pre null
    assert L.moe_expert_ffn_train(fake, fake, None, fake, None, 0, moe.BF16, None, 4, 2, 16, 12, fake, fake, fake, None) == moe.UNSUPPORTED  # H % 8
    assert L.moe_expert_ffn_backward(fake, fake, None, fake, None, fake, fake, 0, moe.BF16, None, 4, 2, 16, 16, fake, 0,
                                     fake, None, None, None, None, None) == moe.WORKSPACE_TOO_SMALL
    assert L.moe_expert_ffn_backward(fake, fake, None, fake, fake + 4, fake, fake, 0, moe.BF16, None, 4, 2, 16, 16, fake, 1 << 30,
                                     fake, None, None, None, None, None) == moe.UNSUPPORTED                            # pre misaligned
    assert L.moe_expert_ffn_backward(fake, fake, None, fake, None, fake, fake, 0, moe.BF16, None, 4, 2, 16, 16, fake, 1 << 30,
                                     None, None, None, None, None, None) == moe.INVALID_ARG                            # nothing asked for
    assert L.moe_decode(fake, moe.F32, fake, fake, None, 8, 16, 4, 1, 2, fake, None) == moe.INVALID_ARG               # gate_w null
    assert L.moe_dynamic_capacity(fake, 8, 4, 1, 1.25, fake, None) == moe.INVALID_ARG      # positive setting: moe_capacity
    assert L.moe_dynamic_capacity(None, 8, 4, 1, 0.0, fake, None) == moe.INVALID_ARG
    assert L.moe_dynamic_capacity(fake, 8, 4, 5, -1.0, fake, None) == moe.INVALID_ARG      # k > E
    assert L.moe_slot_sources(fake, fake, 8, 4, 1, 0, fake, None) == moe.INVALID_ARG       # C < 1
    assert L.moe_slot_sources(fake, None, 8, 4, 1, 2, fake, None) == moe.INVALID_ARG
    assert L.moe_layer_forward(fake, fake, None, fake, None, fake, None, 8, 16, 16, 4, 1, 0.0, 0, 0, moe.F32, fake,
                               None, None, None, None, None, fake, 1 << 30, None, None) == moe.INVALID_ARG            # f <= 0
    assert L.moe_layer_forward(fake, fake, None, fake, None, fake, None, 8, 16, 16, 4, 1, 1.0, 0, 0, moe.F32, fake,
                               None, None, None, None, None, fake, 16, None, None) == moe.WORKSPACE_TOO_SMALL
    dyn = lambda setting, C_max, ws_bytes, router=0, Me=None, bpr=0, C_out=None: L.moe_layer_forward_dynamic(   # noqa: E731
        fake, fake, None, fake, None, fake, None, 64, 16, 16, 4, 2, setting, C_max, 1, 0, moe.F32, router, Me, 8, 0.07, bpr, fake,
        None, None, None, None, None, C_out, fake, ws_bytes, None)
    assert L.moe_layer_dynamic_workspace_bytes(64, 16, 16, 4, 2, 64, moe.F32, 0, 0, 0) > 0
    assert L.moe_layer_dynamic_workspace_bytes(64, 16, 16, 4, 2, 64, moe.F32, 2, 0, 0) == 0                            # unknown router
    assert L.moe_layer_dynamic_workspace_bytes(64, 16, 16, 4, 2, 64, moe.F32, 1, 8, 0) > L.moe_layer_dynamic_workspace_bytes(64, 16, 16, 4, 2, 64, moe.F32, 0, 0, 0)
    assert dyn(0.0, 64, 16) == moe.WORKSPACE_TOO_SMALL
    assert dyn(float("nan"), 64, 1 << 30) == moe.INVALID_ARG
    assert dyn(2.0, 32, 1 << 30) == moe.INVALID_ARG                          # static capacity 64 does not fit buffers sized for 32
    assert dyn(0.0, 0, 1 << 30) == moe.INVALID_ARG
    assert dyn(0.0, 64, 1 << 30, router=1, Me=None) == moe.INVALID_ARG       # cosine router without expert embeddings
    assert dyn(0.0, 64, 1 << 30, C_out=fake + 4) == moe.UNSUPPORTED          # C_out misaligned
    assert L.moe_layer_train_state_bytes(8, 16, 16, 4, 1, 2, moe.F32) > 0
    assert L.moe_layer_train_state_bytes(8, 12, 16, 4, 1, 2, moe.F32) == 0                                             # M % 8
    assert L.moe_layer_forward_train(fake, fake, None, fake, None, fake, None, 8, 16, 16, 4, 1, 1.0, 0, 0, moe.F32, fake,
                                     fake, 16, None) == moe.WORKSPACE_TOO_SMALL
    assert L.moe_layer_forward_train(fake, fake, None, fake, None, fake, None, 8, 16, 16, 4, 1, 1.0, 0, 0, moe.F32, fake,
                                     None, 1 << 30, None) == moe.INVALID_ARG                                           # no state
    assert L.moe_layer_backward(fake, fake, fake, None, fake, 8, 16, 16, 4, 1, 1.0, 0, 0, moe.F32, fake, fake, 16,
                                fake, None, None, None, None, None, None, None) == moe.WORKSPACE_TOO_SMALL
    assert L.moe_layer_backward(fake, fake, fake, None, fake, 8, 16, 16, 4, 1, 1.0, 0, 0, moe.F32, fake, fake, 1 << 30,
                                None, None, None, None, None, None, None, None) == moe.INVALID_ARG                     # dx required


def test_missing_library_fails_loudly(moe, monkeypatch):
    monkeypatch.setattr(moe, "_lib", None)
    monkeypatch.setattr(moe, "LIB_PATH", "/nonexistent/libmoe_mi355x.so")
    with pytest.raises(RuntimeError, match="no fallback"):
        moe.lib()
