"""ctypes binding of libmoe_probe.so, the benchmark's measurement aid (include/moe_mi355x_probe.h)."""
from __future__ import annotations

import ctypes
import os

import torch

PROBE_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libmoe_probe.so")
_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(PROBE_LIB_PATH):
            raise RuntimeError(f"{PROBE_LIB_PATH} is missing: build it with `python -m paper_2206_03382_amd.build`")
        h = ctypes.CDLL(PROBE_LIB_PATH)
        h.moe_probe_mfma_sustained.restype = ctypes.c_int
        h.moe_probe_mfma_sustained.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p,
                                               ctypes.POINTER(ctypes.c_double), ctypes.c_void_p]
        _lib = h
    return _lib


def mfma_sustained_tflops(random_operands: bool = True, seconds: float = 1.0, blocks: int = 256, iters: int = 2000) -> float:
    """Sustained register-only MFMA rate (TFLOP/s) over about `seconds` of back-to-back launches; the last batch is timed."""
    sink = torch.zeros((blocks * 256,), dtype=torch.float32, device="cuda")
    flop = ctypes.c_double()
    stream = torch.cuda.current_stream().cuda_stream

    def launch():
        st = lib().moe_probe_mfma_sustained(blocks, iters, int(random_operands), sink.data_ptr(), ctypes.byref(flop), stream)
        if st != 0:
            raise RuntimeError(f"moe_probe_mfma_sustained: status {st}")

    for _ in range(20):
        launch()
    torch.cuda.synchronize()
    total, last = 0.0, 0.0
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    while total < seconds * 1e3:
        a.record()
        for _ in range(20):
            launch()
        b.record()
        b.synchronize()
        last = a.elapsed_time(b) / 20
        total += last * 20
    return flop.value / (last * 1e-3) / 1e12
