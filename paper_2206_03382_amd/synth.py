"""Seeded synthetic inputs for the MoE-layer hot path (gate -> encode -> expert FFN -> decode).

This module serves both the CPU oracle's tests and the HIP path's tests/bench with the *same bits*.
It holds none of the method's arithmetic: only shapes, random draws, the bf16 storage format, and the
input-side preparation the workloads name (LayerNorm'd tokens, a Zipf-shaped gate bias).

Workloads follow the single-layer shapes the paper sweeps (Sec. 5.1: model/hidden dims in {1024, 2048,
4096}, tokens/step in {4096, 16384, 65536}; Sec. 5.2: 16384 tokens/step, D = H = 2048, top-2) and the
SwinV2-MoE setting (Sec. 5.3: 32 experts, top-1). They stand in for the paper's training data, which is
neither available nor needed: every tensor is drawn from a counter-based generator (Philox) keyed by
(seed, config id, tensor id).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace
from typing import Dict, Optional

import numpy as np

ACT_RELU, ACT_GELU, ACT_SILU = 0, 1, 2
DT_F32, DT_BF16 = 0, 1


@dataclass(frozen=True)
class MoEConfig:
    name: str
    cfg_id: int
    T: int          # tokens per step
    M: int          # model (channel) dim, the paper's D
    H: int          # expert hidden dim
    E: int          # experts
    k: int          # top-k
    f: float        # capacity factor
    act: int
    dtype: int
    normalize: int  # renormalise the k gate weights (1 for k >= 2, 0 for k = 1)
    layernorm: bool = False
    zipf_bias: bool = False

    def scaled(self, **kw) -> "MoEConfig":
        return replace(self, **kw)


CONFIGS = [
    MoEConfig("tiny_fp32", 0, T=1024, M=256, H=512, E=4, k=1, f=1.0, act=ACT_RELU, dtype=DT_F32, normalize=0),
    MoEConfig("mid_bf16", 1, T=16384, M=2048, H=2048, E=8, k=2, f=1.25, act=ACT_GELU, dtype=DT_BF16, normalize=1),
    MoEConfig("vit_bf16", 2, T=25088, M=768, H=3072, E=32, k=1, f=1.25, act=ACT_GELU, dtype=DT_BF16, normalize=0,
              layernorm=True),
    MoEConfig("skewed_bf16", 3, T=65536, M=1024, H=4096, E=64, k=2, f=1.0, act=ACT_GELU, dtype=DT_BF16, normalize=1,
              zipf_bias=True),
    MoEConfig("finegrained_bf16", 4, T=131072, M=4096, H=1024, E=128, k=8, f=2.0, act=ACT_SILU, dtype=DT_BF16,
              normalize=1),
]


# ---- bf16 storage format (round-to-nearest-even truncation of an IEEE fp32) -------------------------------------

def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """fp32 array -> fp32 array whose values are exactly representable in bf16 (RNE). Finite inputs only."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp32 array holding bf16-representable values -> uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    return (u >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# ---- generators -------------------------------------------------------------------------------------------------

def _rng(seed: int, cfg_id: int, tensor_id: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[np.uint64(seed), np.uint64(cfg_id * 64 + tensor_id)]))


def _normal(seed, cfg_id, tensor_id, shape, std) -> np.ndarray:
    a = _rng(seed, cfg_id, tensor_id).standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return a


def _layernorm_rows(x: np.ndarray, eps: float = 1e-5) -> np.ndarray:
    """Per-token LayerNorm without affine parameters, in fp32 (the vision workload's token statistics)."""
    mu = x.mean(axis=1, keepdims=True, dtype=np.float32)
    xc = x - mu
    var = np.mean(xc * xc, axis=1, keepdims=True, dtype=np.float32)
    return (xc / np.sqrt(var + np.float32(eps))).astype(np.float32)


def zipf_gate_bias(E: int, s: float = 1.2, scale: float = 2.0) -> np.ndarray:
    """b_e = scale * ln(w_r), w_r = r^-s / sum_r' r'^-s with rank r = e + 1: a heavy-headed expert popularity."""
    r = np.arange(1, E + 1, dtype=np.float64)
    w = r ** (-s)
    w /= w.sum()
    return (scale * np.log(w)).astype(np.float32)


def make_inputs(cfg: MoEConfig, seed: int = 0, bias_std: float = 0.0) -> Dict[str, Optional[np.ndarray]]:
    """All layer inputs as fp32 arrays; for bf16 configs every value is already bf16-representable.

    x [T,M] ~ N(0,1) (optionally LayerNorm'd), Wg [M,E] ~ N(0,1/M), W1 [E,M,H] ~ N(0,1/M), W2 [E,H,M] ~ N(0,1/H),
    gate_bias [E] (Zipf workload only, fp32), b1 [E,H] / b2 [E,M] ~ N(0, bias_std^2) or None when bias_std == 0.
    """
    T, M, H, E = cfg.T, cfg.M, cfg.H, cfg.E
    c = cfg.cfg_id
    x = _normal(seed, c, 0, (T, M), 1.0)
    if cfg.layernorm:
        x = _layernorm_rows(x)
    Wg = _normal(seed, c, 1, (M, E), 1.0 / math.sqrt(M))
    W1 = _normal(seed, c, 2, (E, M, H), 1.0 / math.sqrt(M))
    W2 = _normal(seed, c, 3, (E, H, M), 1.0 / math.sqrt(H))
    b1 = b2 = None
    if bias_std > 0.0:
        b1 = _normal(seed, c, 4, (E, H), bias_std)
        b2 = _normal(seed, c, 5, (E, M), bias_std)
    if cfg.dtype == DT_BF16:
        x, Wg, W1, W2 = (round_to_bf16(a) for a in (x, Wg, W1, W2))
        if b1 is not None:
            b1, b2 = round_to_bf16(b1), round_to_bf16(b2)
    gate_bias = zipf_gate_bias(E) if cfg.zipf_bias else None
    return dict(x=x, Wg=Wg, gate_bias=gate_bias, W1=W1, b1=b1, W2=W2, b2=b2)


def make_logits(T: int, E: int, seed: int = 0, tensor_id: int = 9, quantum: float = 0.0) -> np.ndarray:
    """fp32 gate logits ~ N(0,1) for gate-only tests; quantum > 0 snaps them to a grid so exact ties occur."""
    a = _normal(seed, 63, tensor_id, (T, E), 1.0)
    if quantum > 0.0:
        a = (np.round(a / np.float32(quantum)) * np.float32(quantum)).astype(np.float32)
    return a
