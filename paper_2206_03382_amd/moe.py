"""Thin ctypes binding of libmoe_mi355x.so: argument marshalling only.

Every step of the path (gate, slot assignment, encode, expert FFN, decode) runs in the library's HIP kernels;
PyTorch is used for device memory and the current stream.  There is no CPU fallback: if the library has not
been built, or no GPU is present, calls raise.
"""
from __future__ import annotations

import ctypes
import os
from typing import Tuple, Dict, Optional, Sequence

import torch

OK, INVALID_ARG, UNSUPPORTED, WORKSPACE_TOO_SMALL, HIP_ERROR, SCRATCH_TOO_SMALL = range(6)
F32, BF16 = 0, 1
ACT_RELU, ACT_GELU, ACT_SILU = 0, 1, 2
ROUTER_LINEAR, ROUTER_COSINE = 0, 1
NUM_STAGE_EVENTS = 7
STAGE_NAMES = ("gate_logits", "gate_topk", "encode", "ffn_gemm1", "ffn_gemm2", "decode")

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libmoe_mi355x.so")

_c = ctypes
_vp, _i64, _i32, _sz, _dbl = _c.c_void_p, _c.c_int64, _c.c_int, _c.c_size_t, _c.c_double

# name -> (restype, argtypes); mirrors include/moe_mi355x.h
SIGNATURES = {
    "moe_status_string": (_c.c_char_p, [_i32]),
    "moe_capacity": (_i64, [_i64, _i64, _i32, _dbl]),
    "moe_gate_workspace_bytes": (_sz, [_i64, _i64, _i32]),
    "moe_layer_workspace_bytes": (_sz, [_i64, _i64, _i64, _i64, _i32, _i64, _i32]),
    "moe_gate_logits": (_i32, [_vp, _vp, _vp, _i32, _i64, _i64, _i64, _vp, _vp]),
    "moe_cosine_gate_workspace_bytes": (_sz, [_i64, _i64, _i64]),
    "moe_gate_logits_cosine": (_i32, [_vp, _vp, _vp, _dbl, _i32, _i64, _i64, _i64, _i64, _vp, _vp, _sz, _vp]),
    "moe_gate_topk": (_i32, [_vp, _i64, _i64, _i32, _i64, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "moe_gate_route_workspace_bytes": (_sz, [_i64, _i64, _i64, _i32, _i32]),
    "moe_gate_route": (_i32, [_vp, _vp, _vp, _i32, _i64, _i64, _i64, _i32, _i64, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "moe_gate_topk_static_max_bytes": (_sz, []),
    "moe_gate_topk_static": (_i32, [_vp, _i64, _i64, _i32, _i64, _i32, _vp, _vp, _vp, _vp, _vp, _vp]),
    "moe_gate_bpr_workspace_bytes": (_sz, [_i64, _i64, _i32]),
    "moe_gate_topk_bpr": (_i32, [_vp, _i64, _i64, _i32, _i64, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "moe_dynamic_capacity": (_i32, [_vp, _i64, _i64, _i32, _dbl, _vp, _vp]),
    "moe_slot_sources": (_i32, [_vp, _vp, _i64, _i64, _i32, _i64, _vp, _vp]),
    "moe_encode": (_i32, [_vp, _i32, _vp, _vp, _vp, _i64, _i64, _i64, _i32, _i64, _vp, _vp]),
    "moe_expert_ffn": (_i32, [_vp, _vp, _vp, _vp, _vp, _i32, _i32, _vp, _i64, _i64, _i64, _i64, _vp, _vp, _vp]),
    "moe_decode": (_i32, [_vp, _i32, _vp, _vp, _vp, _i64, _i64, _i64, _i32, _i64, _vp, _vp]),
    "moe_layer_forward": (_i32, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _i64, _i64, _i64, _i64, _i32, _dbl, _i32, _i32, _i32,
                                 _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp, _c.POINTER(_vp)]),
    "moe_gate_backward_workspace_bytes": (_sz, [_i64, _i64, _i64, _i32]),
    "moe_gate_backward": (_i32, [_vp, _vp, _vp, _vp, _vp, _i32, _i32, _i64, _i64, _i64, _i32, _vp, _sz, _vp, _i32, _vp, _vp, _vp, _vp]),
    "moe_ffn_backward_workspace_bytes": (_sz, [_i64, _i64, _i64, _i64, _i32]),
    "moe_expert_ffn_train": (_i32, [_vp, _vp, _vp, _vp, _vp, _i32, _i32, _vp, _i64, _i64, _i64, _i64, _vp, _vp, _vp, _vp]),
    "moe_expert_ffn_backward": (_i32, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _vp, _i64, _i64, _i64, _i64, _vp, _sz,
                                       _vp, _vp, _vp, _vp, _vp, _vp]),
    "moe_encode_backward": (_i32, [_vp, _i32, _vp, _vp, _i64, _i64, _i64, _i32, _i64, _vp, _vp]),
    "moe_decode_backward": (_i32, [_vp, _vp, _i32, _vp, _vp, _vp, _vp, _i64, _i64, _i64, _i32, _i64, _vp, _vp, _vp]),
    "moe_layer_forward_fused": (_i32, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _i64, _i64, _i64, _i64, _i32, _dbl, _i32, _i32, _i32,
                                       _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp, _c.POINTER(_vp)]),
    "moe_expert_ffn_gather": (_i32, [_vp, _vp, _i64, _vp, _vp, _vp, _vp, _i32, _i32, _vp, _i64, _i64, _i64, _i64, _vp, _vp, _vp]),
    "moe_layer_dynamic_workspace_bytes": (_sz, [_i64, _i64, _i64, _i64, _i32, _i64, _i32, _i32, _i64, _i32]),
    "moe_layer_forward_dynamic": (_i32, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _i64, _i64, _i64, _i64, _i32, _dbl, _i64, _i32, _i32, _i32,
                                         _i32, _vp, _i64, _dbl, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "moe_layer_train_state_bytes": (_sz, [_i64, _i64, _i64, _i64, _i32, _i64, _i32]),
    "moe_layer_forward_train": (_i32, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _i64, _i64, _i64, _i64, _i32, _dbl, _i32, _i32, _i32,
                                       _vp, _vp, _sz, _vp]),
    "moe_layer_backward": (_i32, [_vp, _vp, _vp, _vp, _vp, _i64, _i64, _i64, _i64, _i32, _dbl, _i32, _i32, _i32, _vp, _vp, _sz,
                                  _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "moe_event_create": (_i32, [_c.POINTER(_vp)]),
    "moe_event_destroy": (_i32, [_vp]),
    "moe_event_record": (_i32, [_vp, _vp]),
    "moe_event_synchronize": (_i32, [_vp]),
    "moe_event_elapsed_ms": (_i32, [_vp, _vp, _c.POINTER(_c.c_float)]),
}

_lib = None


class MoEError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {lib().moe_status_string(status).decode()} (status {status})")


def lib() -> ctypes.CDLL:
    """Loads the HIP library on first use; fails loudly if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2206_03382_amd.build` "
                               "(there is no fallback path)")
        handle = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype, fn.argtypes = res, args
        _lib = handle
    return _lib


def _check(status: int, where: str) -> None:
    if status != OK:
        raise MoEError(status, where)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported storage dtype {t.dtype}")


def _p(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("tensors must be contiguous device tensors")
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def capacity(T: int, E: int, k: int, f: float) -> int:
    return int(lib().moe_capacity(T, E, k, float(f)))


def gate_workspace_bytes(T: int, E: int, k: int) -> int:
    return int(lib().moe_gate_workspace_bytes(T, E, k))


def layer_workspace_bytes(T: int, M: int, H: int, E: int, k: int, C: int, dtype: int) -> int:
    return int(lib().moe_layer_workspace_bytes(T, M, H, E, k, C, dtype))


def gate_logits(x: torch.Tensor, Wg: torch.Tensor, gate_bias: Optional[torch.Tensor] = None) -> torch.Tensor:
    T, M = x.shape
    E = Wg.shape[1]
    logits = torch.empty((T, E), dtype=torch.float32, device=x.device)
    _check(lib().moe_gate_logits(_p(x), _p(Wg), _p(gate_bias), _dtype_code(x), T, M, E, _p(logits), _stream()), "moe_gate_logits")
    return logits


def gate_logits_cosine(x: torch.Tensor, Wp: torch.Tensor, Me: torch.Tensor, tau: float) -> torch.Tensor:
    """Cosine-router logits cos(x Wp, Me[e]) / max(tau, 0.01); Wp [M,D] in x's dtype, Me [E,D] fp32."""
    T, M = x.shape
    D = Wp.shape[1]
    E = Me.shape[0]
    nbytes = int(lib().moe_cosine_gate_workspace_bytes(T, D, E))
    if nbytes == 0:
        raise MoEError(UNSUPPORTED, "moe_cosine_gate_workspace_bytes")
    ws = torch.empty((nbytes,), dtype=torch.uint8, device=x.device)
    logits = torch.empty((T, E), dtype=torch.float32, device=x.device)
    _check(lib().moe_gate_logits_cosine(_p(x), _p(Wp), _p(Me), float(tau), _dtype_code(x), T, M, D, E, _p(logits), _p(ws),
                                        ws.numel(), _stream()), "moe_gate_logits_cosine")
    return logits


def gate_topk(logits: torch.Tensor, k: int, C: int, normalize: int, want_slot_src: bool = True,
              bpr: bool = False) -> Dict[str, torch.Tensor]:
    """Top-k, gate weights and slot assignment; bpr: batch prioritized routing order instead of token order."""
    T, E = logits.shape
    dev = logits.device
    idx = torch.empty((T, k), dtype=torch.int32, device=dev)
    loc = torch.empty((T, k), dtype=torch.int32, device=dev)
    gate_w = torch.empty((T, k), dtype=torch.float32, device=dev)
    counts = torch.empty((E,), dtype=torch.int32, device=dev)
    slot_src = torch.empty((E, C), dtype=torch.int32, device=dev) if want_slot_src else None
    nbytes = int(lib().moe_gate_bpr_workspace_bytes(T, E, k)) if bpr else gate_workspace_bytes(T, E, k)
    if bpr and nbytes == 0:
        raise MoEError(UNSUPPORTED, "moe_gate_bpr_workspace_bytes")
    ws = torch.empty((max(nbytes, 16),), dtype=torch.uint8, device=dev)
    entry = lib().moe_gate_topk_bpr if bpr else lib().moe_gate_topk
    _check(entry(_p(logits), T, E, k, C, int(normalize), _p(idx), _p(gate_w), _p(loc), _p(counts), _p(slot_src),
                 _p(ws), ws.numel(), _stream()), "moe_gate_topk_bpr" if bpr else "moe_gate_topk")
    return dict(idx=idx, loc=loc, gate_w=gate_w, counts=counts, slot_src=slot_src)


def gate_route(x: torch.Tensor, Wg: torch.Tensor, gate_bias: Optional[torch.Tensor], k: int, C: int, normalize: int) -> Dict[str, torch.Tensor]:
    """The gate from the tokens (moe_gate_route): logits, idx, gate_w, loc, counts, slot_src."""
    T, M = x.shape
    E = Wg.shape[1]
    dev = x.device
    code = _dtype_code(x)
    nbytes = int(lib().moe_gate_route_workspace_bytes(T, M, E, k, code))
    if nbytes == 0:
        raise MoEError(UNSUPPORTED, "moe_gate_route_workspace_bytes")
    ws = torch.empty((nbytes,), dtype=torch.uint8, device=dev)
    r = dict(logits=torch.empty((T, E), dtype=torch.float32, device=dev), idx=torch.empty((T, k), dtype=torch.int32, device=dev),
             loc=torch.empty((T, k), dtype=torch.int32, device=dev), gate_w=torch.empty((T, k), dtype=torch.float32, device=dev),
             counts=torch.empty((E,), dtype=torch.int32, device=dev), slot_src=torch.empty((E, C), dtype=torch.int32, device=dev))
    _check(lib().moe_gate_route(_p(x), _p(Wg), _p(gate_bias), code, T, M, E, k, C, int(normalize), _p(r["logits"]), _p(r["idx"]),
                                _p(r["gate_w"]), _p(r["loc"]), _p(r["counts"]), _p(r["slot_src"]), _p(ws), ws.numel(), _stream()),
           "moe_gate_route")
    return r


def gate_topk_static(logits: torch.Tensor, k: int, C: int, normalize: int, out: Dict[str, torch.Tensor]) -> Dict[str, torch.Tensor]:
    """moe_gate_topk_static into caller-provided outputs (idx, loc, gate_w, counts, slot_src): nothing is allocated."""
    T, E = logits.shape
    _check(lib().moe_gate_topk_static(_p(logits), T, E, k, C, int(normalize), _p(out["idx"]), _p(out["gate_w"]), _p(out["loc"]),
                                      _p(out["counts"]), _p(out.get("slot_src")), _stream()), "moe_gate_topk_static")
    return out


def dynamic_capacity(counts: torch.Tensor, T: int, k: int, capacity_setting: float) -> Tuple[int, int]:
    """(capacity to use, needed capacity) for capacity_setting <= 0; reads two integers back from the device."""
    E = counts.shape[0]
    out = torch.empty((2,), dtype=torch.int64, device=counts.device)
    _check(lib().moe_dynamic_capacity(_p(counts), T, E, k, float(capacity_setting), _p(out), _stream()), "moe_dynamic_capacity")
    C, needed = out.cpu().tolist()
    return int(C), int(needed)


def slot_sources(idx: torch.Tensor, loc: torch.Tensor, E: int, C: int) -> torch.Tensor:
    T, k = idx.shape
    slot_src = torch.empty((E, C), dtype=torch.int32, device=idx.device)
    _check(lib().moe_slot_sources(_p(idx), _p(loc), T, E, k, C, _p(slot_src), _stream()), "moe_slot_sources")
    return slot_src


class DynamicLayer:
    """The layer with the dynamic capacity factor through moe_layer_forward_dynamic: owns workspace and outputs sized for
    C_max, so that `forward` allocates nothing and never synchronises (the chosen capacity stays on the device)."""

    def __init__(self, Wg, gate_bias, W1, b1, W2, b2, T: int, k: int, capacity_setting: float, normalize: int, act: int,
                 C_max: Optional[int] = None, bpr: bool = False, cosine_Me: Optional[torch.Tensor] = None, cosine_tau: float = 0.07):
        self.Wg, self.gate_bias, self.W1, self.b1, self.W2, self.b2 = Wg, gate_bias, W1, b1, W2, b2
        self.E, self.M, self.H = W1.shape
        self.T, self.k, self.setting, self.normalize, self.act = T, k, float(capacity_setting), int(normalize), int(act)
        self.C_max = int(T if C_max is None else C_max)
        self.bpr = int(bool(bpr))
        self.Me, self.tau = cosine_Me, float(cosine_tau)
        self.router = ROUTER_LINEAR if cosine_Me is None else ROUTER_COSINE
        self.D = 0 if cosine_Me is None else int(cosine_Me.shape[1])
        self.dtype = _dtype_code(W1)
        nbytes = int(lib().moe_layer_dynamic_workspace_bytes(T, self.M, self.H, self.E, k, self.C_max, self.dtype, self.router, self.D, self.bpr))
        if nbytes == 0:
            raise MoEError(UNSUPPORTED, "moe_layer_dynamic_workspace_bytes")
        dev = W1.device
        self.ws = torch.empty((nbytes,), dtype=torch.uint8, device=dev)
        self.out = torch.empty((T, self.M), dtype=W1.dtype, device=dev)
        self.routing = dict(idx=torch.empty((T, k), dtype=torch.int32, device=dev), loc=torch.empty((T, k), dtype=torch.int32, device=dev),
                            gate_w=torch.empty((T, k), dtype=torch.float32, device=dev),
                            counts=torch.empty((self.E,), dtype=torch.int32, device=dev),
                            logits=torch.empty((T, self.E), dtype=torch.float32, device=dev),
                            C=torch.empty((2,), dtype=torch.int64, device=dev))

    def forward(self, x: torch.Tensor) -> torch.Tensor:
        r = self.routing
        _check(lib().moe_layer_forward_dynamic(_p(x), _p(self.Wg), _p(self.gate_bias), _p(self.W1), _p(self.b1), _p(self.W2), _p(self.b2),
                                               self.T, self.M, self.H, self.E, self.k, self.setting, self.C_max, self.normalize,
                                               self.act, self.dtype, self.router, _p(self.Me), self.D, self.tau, self.bpr,
                                               _p(self.out), _p(r["idx"]), _p(r["loc"]), _p(r["gate_w"]), _p(r["counts"]),
                                               _p(r["logits"]), _p(r["C"]), _p(self.ws), self.ws.numel(), _stream()),
               "moe_layer_forward_dynamic")
        return self.out


def layer_forward_dynamic(x, Wg, gate_bias, W1, b1, W2, b2, k: int, capacity_setting: float, normalize: int, act: int,
                          C_max: Optional[int] = None, bpr: bool = False, cosine_Me: Optional[torch.Tensor] = None,
                          cosine_tau: float = 0.07) -> Dict[str, torch.Tensor]:
    """One call of moe_layer_forward_dynamic; the chosen and the needed capacity are read back afterwards for the caller."""
    layer = DynamicLayer(Wg, gate_bias, W1, b1, W2, b2, x.shape[0], k, capacity_setting, normalize, act, C_max, bpr, cosine_Me, cosine_tau)
    out = layer.forward(x)
    r = dict(layer.routing)
    C, needed = r.pop("C").cpu().tolist()
    r.update(C=int(C), needed_capacity=int(needed), out=out)
    return r


def encode(x: torch.Tensor, idx: torch.Tensor, loc: torch.Tensor, slot_src: Optional[torch.Tensor], E: int, C: int) -> torch.Tensor:
    T, M = x.shape
    k = idx.shape[1]
    Z = torch.empty((E, C, M), dtype=x.dtype, device=x.device)
    _check(lib().moe_encode(_p(x), _dtype_code(x), _p(idx), _p(loc), _p(slot_src), T, M, E, k, C, _p(Z), _stream()), "moe_encode")
    return Z


def expert_ffn(Z: torch.Tensor, W1: torch.Tensor, b1: Optional[torch.Tensor], W2: torch.Tensor, b2: Optional[torch.Tensor],
               act: int, counts: Optional[torch.Tensor] = None, Y: Optional[torch.Tensor] = None,
               hidden: Optional[torch.Tensor] = None) -> torch.Tensor:
    E, C, M = Z.shape
    H = W1.shape[2]
    if Y is None:
        Y = torch.empty((E, C, M), dtype=Z.dtype, device=Z.device)
    if hidden is None:
        hidden = torch.empty((E, C, H), dtype=Z.dtype, device=Z.device)
    _check(lib().moe_expert_ffn(_p(Z), _p(W1), _p(b1), _p(W2), _p(b2), act, _dtype_code(Z), _p(counts), E, C, M, H,
                                _p(hidden), _p(Y), _stream()), "moe_expert_ffn")
    return Y


def expert_ffn_gather(x: torch.Tensor, slot_src: torch.Tensor, W1: torch.Tensor, b1: Optional[torch.Tensor], W2: torch.Tensor,
                      b2: Optional[torch.Tensor], act: int, counts: Optional[torch.Tensor] = None) -> torch.Tensor:
    """encode + expert_ffn in one: the first GEMM reads row c of expert e from x[slot_src[e, c]]."""
    T, M = x.shape
    E, C = slot_src.shape
    H = W1.shape[2]
    Y = torch.empty((E, C, M), dtype=x.dtype, device=x.device)
    hidden = torch.empty((E, C, H), dtype=x.dtype, device=x.device)
    _check(lib().moe_expert_ffn_gather(_p(x), _p(slot_src), T, _p(W1), _p(b1), _p(W2), _p(b2), act, _dtype_code(x), _p(counts),
                                       E, C, M, H, _p(hidden), _p(Y), _stream()), "moe_expert_ffn_gather")
    return Y


def decode(Y: torch.Tensor, idx: torch.Tensor, loc: torch.Tensor, gate_w: torch.Tensor) -> torch.Tensor:
    E, C, M = Y.shape
    T, k = idx.shape
    out = torch.empty((T, M), dtype=Y.dtype, device=Y.device)
    _check(lib().moe_decode(_p(Y), _dtype_code(Y), _p(idx), _p(loc), _p(gate_w), T, M, E, k, C, _p(out), _stream()), "moe_decode")
    return out


def gate_backward(x: torch.Tensor, Wg: torch.Tensor, logits: torch.Tensor, idx: torch.Tensor, dgate_w: torch.Tensor, normalize: int,
                  dx: Optional[torch.Tensor] = None) -> Dict[str, torch.Tensor]:
    """dlogits, dx (added to `dx` if given), dWg, dbias of the gate."""
    T, M = x.shape
    E = Wg.shape[1]
    k = idx.shape[1]
    nbytes = int(lib().moe_gate_backward_workspace_bytes(T, M, E, k))
    if nbytes == 0:
        raise MoEError(UNSUPPORTED, "moe_gate_backward_workspace_bytes")
    ws = torch.empty((nbytes,), dtype=torch.uint8, device=x.device)
    accumulate = dx is not None
    if dx is None:
        dx = torch.empty_like(x)
    g = dict(dx=dx, dWg=torch.empty_like(Wg), dbias=torch.empty((E,), dtype=torch.float32, device=x.device),
             dlogits=torch.empty((T, E), dtype=torch.float32, device=x.device))
    _check(lib().moe_gate_backward(_p(x), _p(Wg), _p(logits), _p(idx), _p(dgate_w), int(normalize), _dtype_code(x), T, M, E, k,
                                   _p(ws), ws.numel(), _p(g["dx"]), int(accumulate), _p(g["dWg"]), _p(g["dbias"]), _p(g["dlogits"]),
                                   _stream()), "moe_gate_backward")
    return g


def expert_ffn_train(Z: torch.Tensor, W1: torch.Tensor, b1: Optional[torch.Tensor], W2: torch.Tensor, b2: Optional[torch.Tensor],
                     act: int, counts: Optional[torch.Tensor] = None):
    """moe_expert_ffn that also keeps the pre-activations; returns (Y, hidden, pre)."""
    E, C, M = Z.shape
    H = W1.shape[2]
    Y = torch.empty((E, C, M), dtype=Z.dtype, device=Z.device)
    hidden = torch.empty((E, C, H), dtype=Z.dtype, device=Z.device)
    pre = torch.empty((E, C, H), dtype=Z.dtype, device=Z.device)
    _check(lib().moe_expert_ffn_train(_p(Z), _p(W1), _p(b1), _p(W2), _p(b2), act, _dtype_code(Z), _p(counts), E, C, M, H,
                                      _p(pre), _p(hidden), _p(Y), _stream()), "moe_expert_ffn_train")
    return Y, hidden, pre


def expert_ffn_backward(Z: torch.Tensor, W1: torch.Tensor, b1: Optional[torch.Tensor], W2: torch.Tensor, hidden: torch.Tensor,
                        dY: torch.Tensor, act: int, counts: Optional[torch.Tensor] = None,
                        pre: Optional[torch.Tensor] = None) -> Dict[str, torch.Tensor]:
    """dZ, dW1, db1, dW2, db2 of the expert layer; `hidden` is the activation buffer moe_expert_ffn filled, `pre` the
    pre-activations moe_expert_ffn_train kept (recomputed when None)."""
    E, C, M = Z.shape
    H = W1.shape[2]
    code = _dtype_code(Z)
    nbytes = int(lib().moe_ffn_backward_workspace_bytes(E, C, M, H, code))
    if nbytes == 0:
        raise MoEError(UNSUPPORTED, "moe_ffn_backward_workspace_bytes")
    ws = torch.empty((nbytes,), dtype=torch.uint8, device=Z.device)
    g = dict(dZ=torch.zeros_like(Z), dW1=torch.empty_like(W1), db1=torch.empty((E, H), dtype=Z.dtype, device=Z.device),
             dW2=torch.empty_like(W2), db2=torch.empty((E, M), dtype=Z.dtype, device=Z.device))
    _check(lib().moe_expert_ffn_backward(_p(Z), _p(W1), _p(b1), _p(W2), _p(pre), _p(hidden), _p(dY), act, code, _p(counts), E, C, M, H,
                                         _p(ws), ws.numel(), _p(g["dZ"]), _p(g["dW1"]), _p(g["db1"]), _p(g["dW2"]), _p(g["db2"]),
                                         _stream()), "moe_expert_ffn_backward")
    return g


def encode_backward(dZ: torch.Tensor, idx: torch.Tensor, loc: torch.Tensor) -> torch.Tensor:
    E, C, M = dZ.shape
    T, k = idx.shape
    dx = torch.empty((T, M), dtype=dZ.dtype, device=dZ.device)
    _check(lib().moe_encode_backward(_p(dZ), _dtype_code(dZ), _p(idx), _p(loc), T, M, E, k, C, _p(dx), _stream()), "moe_encode_backward")
    return dx


def decode_backward(d_out: torch.Tensor, Y: torch.Tensor, idx: torch.Tensor, loc: torch.Tensor, gate_w: torch.Tensor,
                    slot_src: torch.Tensor) -> Tuple[torch.Tensor, torch.Tensor]:
    """(dY [E,C,M], dgate_w [T,k])."""
    E, C, M = Y.shape
    T, k = idx.shape
    dY = torch.empty_like(Y)
    dgate_w = torch.empty((T, k), dtype=torch.float32, device=Y.device)
    _check(lib().moe_decode_backward(_p(d_out), _p(Y), _dtype_code(Y), _p(idx), _p(loc), _p(gate_w), _p(slot_src), T, M, E, k, C,
                                     _p(dY), _p(dgate_w), _stream()), "moe_decode_backward")
    return dY, dgate_w


def layer_forward_backward(x, Wg, gate_bias, W1, b1, W2, b2, k: int, f: float, normalize: int, act: int,
                           d_out: torch.Tensor) -> Dict[str, torch.Tensor]:
    """One training pass of the layer through the separate entry points: forward (keeping what the backward needs), then
    the backward of decode, of the experts, of encode and of the gate.  Returns out and all gradients."""
    T, E = x.shape[0], W1.shape[0]
    C = capacity(T, E, k, f)
    r = gate_route(x, Wg, gate_bias, k, C, normalize)
    logits = r["logits"]
    Z = encode(x, r["idx"], r["loc"], r["slot_src"], E, C)
    Y, hidden, pre = expert_ffn_train(Z, W1, b1, W2, b2, act, counts=r["counts"])
    out = decode(Y, r["idx"], r["loc"], r["gate_w"])
    dY, dgate_w = decode_backward(d_out, Y, r["idx"], r["loc"], r["gate_w"], r["slot_src"])
    g = expert_ffn_backward(Z, W1, b1, W2, hidden, dY, act, counts=r["counts"], pre=pre)
    dx = encode_backward(g["dZ"], r["idx"], r["loc"])
    gg = gate_backward(x, Wg, logits, r["idx"], dgate_w, normalize, dx=dx)
    return dict(out=out, dx=gg["dx"], dWg=gg["dWg"], dgate_bias=gg["dbias"], dW1=g["dW1"], db1=g["db1"], dW2=g["dW2"],
                db2=g["db2"], routing=r, logits=logits)


class TrainLayer:
    """One MoE layer's training step through moe_layer_forward_train / moe_layer_backward; owns the state buffer."""

    def __init__(self, Wg, gate_bias, W1, b1, W2, b2, T: int, k: int, f: float, normalize: int, act: int):
        self.Wg, self.gate_bias, self.W1, self.b1, self.W2, self.b2 = Wg, gate_bias, W1, b1, W2, b2
        self.T, self.k, self.f, self.normalize, self.act = T, k, f, int(normalize), act
        self.E, self.M, self.H = W1.shape
        self.C = capacity(T, self.E, k, f)
        self.code = _dtype_code(W1)
        nbytes = int(lib().moe_layer_train_state_bytes(T, self.M, self.H, self.E, k, self.C, self.code))
        if nbytes == 0:
            raise MoEError(UNSUPPORTED, "moe_layer_train_state_bytes")
        self.state = torch.empty((nbytes,), dtype=torch.uint8, device=W1.device)

    def forward(self, x: torch.Tensor) -> torch.Tensor:
        out = torch.empty_like(x)
        _check(lib().moe_layer_forward_train(_p(x), _p(self.Wg), _p(self.gate_bias), _p(self.W1), _p(self.b1), _p(self.W2),
                                             _p(self.b2), self.T, self.M, self.H, self.E, self.k, self.f, self.normalize,
                                             self.act, self.code, _p(out), _p(self.state), self.state.numel(), _stream()),
               "moe_layer_forward_train")
        return out

    def backward(self, x: torch.Tensor, d_out: torch.Tensor, grads: Optional[Dict[str, torch.Tensor]] = None) -> Dict[str, torch.Tensor]:
        g = grads
        if g is None:
            dev, dt = x.device, x.dtype
            g = dict(dx=torch.empty_like(x), dWg=torch.empty_like(self.Wg), dgate_bias=torch.empty((self.E,), dtype=torch.float32, device=dev),
                     dW1=torch.empty_like(self.W1), db1=torch.empty((self.E, self.H), dtype=dt, device=dev),
                     dW2=torch.empty_like(self.W2), db2=torch.empty((self.E, self.M), dtype=dt, device=dev))
        _check(lib().moe_layer_backward(_p(x), _p(self.Wg), _p(self.W1), _p(self.b1), _p(self.W2), self.T, self.M, self.H, self.E,
                                        self.k, self.f, self.normalize, self.act, self.code, _p(d_out), _p(self.state),
                                        self.state.numel(), _p(g["dx"]), _p(g["dWg"]), _p(g["dgate_bias"]), _p(g["dW1"]),
                                        _p(g["db1"]), _p(g["dW2"]), _p(g["db2"]), _stream()), "moe_layer_backward")
        return g


class StageEvents:
    """MOE_NUM_STAGE_EVENTS HIP events, recorded by moe_layer_forward on its stream at the stage boundaries."""

    def __init__(self):
        self.handles = (_vp * NUM_STAGE_EVENTS)()
        for i in range(NUM_STAGE_EVENTS):
            ev = _vp()
            _check(lib().moe_event_create(ctypes.byref(ev)), "moe_event_create")
            self.handles[i] = ev

    def stage_ms(self) -> Sequence[float]:
        _check(lib().moe_event_synchronize(self.handles[NUM_STAGE_EVENTS - 1]), "moe_event_synchronize")
        out = []
        for i in range(NUM_STAGE_EVENTS - 1):
            ms = ctypes.c_float()
            _check(lib().moe_event_elapsed_ms(self.handles[i], self.handles[i + 1], ctypes.byref(ms)), "moe_event_elapsed_ms")
            out.append(ms.value)
        return out

    def close(self):
        for h in self.handles:
            if h:
                lib().moe_event_destroy(h)
        self.handles = (_vp * NUM_STAGE_EVENTS)()


class MoELayer:
    """Holds the layer's parameters, output and workspace so that `forward` allocates nothing."""

    def __init__(self, Wg, gate_bias, W1, b1, W2, b2, T: int, k: int, f: float, normalize: int, act: int,
                 keep_routing: bool = False):
        self.Wg, self.gate_bias, self.W1, self.b1, self.W2, self.b2 = Wg, gate_bias, W1, b1, W2, b2
        self.E, self.M, self.H = W1.shape
        self.T, self.k, self.f, self.normalize, self.act = T, k, float(f), int(normalize), int(act)
        self.dtype = _dtype_code(W1)
        self.C = capacity(T, self.E, k, f)
        if self.C < 1:
            raise MoEError(INVALID_ARG, "moe_capacity")
        nbytes = layer_workspace_bytes(T, self.M, self.H, self.E, k, self.C, self.dtype)
        if nbytes == 0:
            raise MoEError(UNSUPPORTED, "moe_layer_workspace_bytes")
        dev = W1.device
        self.ws = torch.empty((nbytes,), dtype=torch.uint8, device=dev)
        self.out = torch.empty((T, self.M), dtype=W1.dtype, device=dev)
        self.routing = None
        if keep_routing:
            self.routing = dict(idx=torch.empty((T, k), dtype=torch.int32, device=dev),
                                loc=torch.empty((T, k), dtype=torch.int32, device=dev),
                                gate_w=torch.empty((T, k), dtype=torch.float32, device=dev),
                                counts=torch.empty((self.E,), dtype=torch.int32, device=dev),
                                logits=torch.empty((T, self.E), dtype=torch.float32, device=dev))

    def forward(self, x: torch.Tensor, events: Optional[StageEvents] = None, fuse_dispatch: bool = False) -> torch.Tensor:
        """One pass of the layer.  fuse_dispatch: let the first expert GEMM gather its rows from x (no dispatch buffer)."""
        if tuple(x.shape) != (self.T, self.M) or _dtype_code(x) != self.dtype:
            raise ValueError(f"x must be [{self.T}, {self.M}] in the layer's storage dtype")
        r = self.routing or {}
        ev = events.handles if events is not None else None
        entry = lib().moe_layer_forward_fused if fuse_dispatch else lib().moe_layer_forward
        _check(entry(_p(x), _p(self.Wg), _p(self.gate_bias), _p(self.W1), _p(self.b1), _p(self.W2), _p(self.b2),
                     self.T, self.M, self.H, self.E, self.k, self.f, self.normalize, self.act, self.dtype,
                     _p(self.out), _p(r.get("idx")), _p(r.get("loc")), _p(r.get("gate_w")), _p(r.get("counts")),
                     _p(r.get("logits")), _p(self.ws), self.ws.numel(), _stream(), ev), "moe_layer_forward")
        return self.out
