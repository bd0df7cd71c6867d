"""CPU oracle for the single-GPU hot path of a Tutel-style MoE layer.  TEST INFRASTRUCTURE ONLY.

Nothing in the product path may import this file: only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline
leg use it.  It shares no code with the HIP library and never receives a value computed by it.

What it computes (arXiv 2206.03382):
  * Sec. 2.1 (background, Fig. 2): gating function -> dispatch -> expert feed-forward layer -> combine.
  * Sec. 2.1, Eq. 1: expert capacity  C = k * f * T / E  (rounded up here; the paper states no rounding).
  * Sec. 2.1 "MoE Frameworks": the routing logic is GShard's, kept unchanged: deterministic, order-based
    truncation at capacity.
  * Appendix B (the dense-vs-sparse figure and the text around it): encode/decode are, by definition, contractions with a
    one-hot [T, E, C] mask; the sparse form only skips the multiplications by zero.  The *dense* form is the
    definition and is what `encode_dense` / `decode_dense` write out.  `encode_sparse` / `decode_sparse` are the
    same sums with the zero terms skipped (used where the [T, E, C] mask would not fit in memory).

Precision: every floating-point step is fp64, with one exception that the method fixes: the gate logits are
rounded once to fp32, because top-k selection (an integer decision) is taken on fp32 logits with ties going to
the lower expert index.  Softmax, gate weights, FFN and combine are fp64 on the fp32 logits / the given inputs.

Readings where the paper is silent (each listed again in the design notes):
  R1  C = ceil(k*f*T/E) evaluated left to right in double.
  R2  gate = linear layer (x @ Wg + bias) -> softmax over all E experts; top-k chosen on the fp32 logits.
  R3  ties -> lower expert index; -0.0 == +0.0.
  R4  arrival order at an expert = (choice rank j ascending, token t ascending); `loc` is the 0-based arrival
      position counted over ALL arrivals (so a dropped choice has loc >= C); kept <=> loc < C.
  R5  gate weight of choice j = p[t, idx[t,j]]; with normalize=1 it is divided by the sum over all k choices
      (kept or dropped alike).
  R6  encode copies rows unscaled; only decode applies the gate weight.  Unfilled slots are zero.
  R7  activations: ReLU; GeLU = 0.5 x (1 + erf(x / sqrt 2)); SiLU = x / (1 + exp(-x)).
  R8  a token whose choices were all dropped gets an all-zero output row.
  R9  storage precision (bf16 workloads): the oracle takes the bf16 inputs as exact values and never rounds an
      intermediate; what the device path rounds (hidden activations, expert outputs, the final sum) is absorbed by the
      output tolerance.
  R10 rows of unfilled slots carry no information: they are zero in Z and are not computed by the zero-skipping tiers.
  R11 the gate's dot products are summed in fp64 and rounded once to fp32, so that the integer decisions taken on them
      do not depend on a summation order.
  R12 workload preparation (LayerNorm'd tokens, Zipf gate bias) belongs to the input generator, not to the method.
  R13 dynamic capacity (Sec. 4.1 "Dynamic Capacity Factor", capacity_setting x): x > 0 is the factor f itself;
      x = 0 means the smallest capacity that drops nothing, which is the arrival count of the fullest expert
      (Eq. 1 with the smallest such factor gives exactly that integer); x < 0 the same but never above the
      capacity that factor -x gives.
  R14 backward of encode / decode (Appendix B, the differentiable fast encode and decode operators; the figure with
      the formulas is lost): the plain derivatives of the dense contractions.  encode is not scaled by the gate
      weight here (R6), so its backward has no gate-weight gradient; idx and loc carry no gradient.
  R15 cosine router (Appendix, "A New Cosine Router", its Eq.): logits[t,e] = cos(W x_t, M_e) / tau with the
      temperature clamped below at 0.01; the projection W x (dimension D) is rounded once to fp32 like the linear
      gate's logits; norms are clamped below at 1e-12 (the paper gives no epsilon); the rest of the gate is unchanged.
  R16 batch prioritized routing (named in Sec. 3.2 and the Appendix's routing ablation, defined in the work cited
      there): slots are handed out in order of decreasing token priority instead of token order, rank j still
      outermost; priority = the token's largest routing probability max_e p[t,e], rounded to fp32 (the comparison
      is an integer-like decision, so both sides take it on the same fp32 key); equal priorities -> lower token.
  R17 backward of the expert feed-forward layer (Sec. 3.2: the backward pass runs "the backward computation of the
      expert"): the chain rule through y = act(z W1 + b1) W2 + b2, rows past an expert's fill contributing nothing;
      ReLU'(0) = 0.
  R18 backward of the gate (the paper only says the backward pass mirrors the forward, Sec. 3.2): the chain rule through
      gate weight = (optionally renormalised) softmax probability at the chosen experts, and through the linear layer;
      the choice of experts and the slot assignment are integer decisions and carry no gradient.

Pins (tests/test_oracle_*.py): Eq. 1 closed forms; the Fig. 2 worked shape; a hand-worked routing example;
exhaustive/brute-force sequential-arrival simulation; invariants; tie cases; special cases that reduce to
torch's linear/softmax/topk/activation routines; dense == sparse == streamed.  No function here is "parity unpinned".
"""
from __future__ import annotations

import math
from typing import Dict, Optional, Sequence

import numpy as np
from scipy.special import erf as _erf

ACT_RELU, ACT_GELU, ACT_SILU = 0, 1, 2


# ---------------------------------------------------------------------------------------------------------------
# Eq. 1 (Sec. 2.1): expert capacity
# ---------------------------------------------------------------------------------------------------------------

def capacity(T: int, E: int, k: int, f: float) -> int:
    """C = ceil(k * f * T / E), evaluated left to right in double (reading R1)."""
    return int(math.ceil(float(k) * float(f) * float(T) / float(E)))


def dynamic_capacity(counts: np.ndarray, T: int, E: int, k: int, capacity_setting: float) -> int:
    """Capacity under the dynamic capacity factor of Sec. 4.1 (reading R13); `counts` are the un-truncated arrivals."""
    x = float(capacity_setting)
    if x > 0:
        return capacity(T, E, k, x)
    needed = int(np.max(np.asarray(counts)))          # the fullest expert decides: nothing is dropped iff C >= this
    if x == 0:
        return needed
    return min(needed, capacity(T, E, k, -x))


# ---------------------------------------------------------------------------------------------------------------
# Gating function (Sec. 2.1; reading R2/R3)
# ---------------------------------------------------------------------------------------------------------------

def gate_logits(x: np.ndarray, Wg: np.ndarray, bias: Optional[np.ndarray] = None, rows_per_pass: int = 8192) -> np.ndarray:
    """logits[t,e] = sum_m x[t,m] Wg[m,e] + bias[e], summed in fp64 and rounded once to fp32.

    Token rows are independent, so they are processed `rows_per_pass` at a time only to bound memory.
    """
    T = x.shape[0]
    Wd = np.asarray(Wg, dtype=np.float64)
    out = np.empty((T, Wd.shape[1]), dtype=np.float32)
    bd = None if bias is None else np.asarray(bias, dtype=np.float64)
    for s in range(0, T, rows_per_pass):
        acc = np.asarray(x[s:s + rows_per_pass], dtype=np.float64) @ Wd
        if bd is not None:
            acc = acc + bd[None, :]
        out[s:s + rows_per_pass] = acc.astype(np.float32)
    return out


def cosine_gate_logits(x: np.ndarray, Wp: np.ndarray, Me: np.ndarray, tau: float, rows_per_pass: int = 8192) -> np.ndarray:
    """Cosine router (Appendix, "A New Cosine Router"; reading R15): cos(x Wp, Me[e]) / max(tau, 0.01) in fp64 on the
    fp32-rounded projection, rounded once to fp32.   x [T,M], Wp [M,D] (the projection, stored input-major), Me [E,D]."""
    proj = gate_logits(x, Wp, None, rows_per_pass).astype(np.float64)          # x Wp: fp64 sums, one rounding to fp32
    Md = np.asarray(Me, dtype=np.float64)
    nx = np.maximum(np.sqrt((proj * proj).sum(axis=1)), 1e-12)
    ne = np.maximum(np.sqrt((Md * Md).sum(axis=1)), 1e-12)
    cos = (proj @ Md.T) / (nx[:, None] * ne[None, :])
    return (cos / max(float(tau), 0.01)).astype(np.float32)


def softmax_rows(logits: np.ndarray) -> np.ndarray:
    """p[t,:] = softmax over all E experts of the fp32 logits, in fp64 (max-subtracted)."""
    z = np.asarray(logits, dtype=np.float32).astype(np.float64)
    z = z - z.max(axis=1, keepdims=True)
    e = np.exp(z)
    return e / e.sum(axis=1, keepdims=True)


def topk_experts(logits: np.ndarray, k: int) -> np.ndarray:
    """idx[t,j] = the j-th largest fp32 logit of token t; equal logits -> lower expert index first (R3).

    k rounds of argmax with the already chosen experts masked out; numpy's argmax returns the first maximum.
    """
    work = np.array(logits, dtype=np.float32, copy=True)
    T, E = work.shape
    assert 1 <= k <= E
    assert np.isfinite(work).all(), "routing is undefined for non-finite logits"
    rows = np.arange(T)
    idx = np.empty((T, k), dtype=np.int32)
    for j in range(k):
        idx[:, j] = np.argmax(work, axis=1)
        work[rows, idx[:, j]] = -np.inf
    return idx


def gate_weights(p: np.ndarray, idx: np.ndarray, normalize: int) -> np.ndarray:
    """w[t,j] = p[t, idx[t,j]], optionally divided by the sum over the token's k choices (R5). fp64."""
    T = idx.shape[0]
    w = p[np.arange(T)[:, None], idx]
    if normalize:
        w = w / w.sum(axis=1, keepdims=True)
    return w


def gate_backward(logits: np.ndarray, idx: np.ndarray, dgate_w: np.ndarray, normalize: int) -> np.ndarray:
    """d loss / d logits given d loss / d gate_w (reading R18), fp64.

    Forward: p = softmax(logits); g[t,j] = p[t, idx[t,j]]; gate_w = g / sum_j g if normalize else g.
    """
    p = softmax_rows(logits)
    T, E = p.shape
    rows = np.arange(T)[:, None]
    g = p[rows, idx]
    dw = np.asarray(dgate_w, dtype=np.float64)
    if normalize:
        S = g.sum(axis=1, keepdims=True)
        w = g / S
        dg = (dw - (dw * w).sum(axis=1, keepdims=True)) / S
    else:
        dg = dw
    dp = np.zeros((T, E), dtype=np.float64)
    np.add.at(dp, (np.broadcast_to(rows, idx.shape), idx), dg)
    return p * (dp - (p * dp).sum(axis=1, keepdims=True))      # softmax Jacobian applied to dp


def gate_logits_backward(x: np.ndarray, Wg: np.ndarray, dlogits: np.ndarray) -> Dict[str, np.ndarray]:
    """Backward of logits = x Wg + bias: dx = dlogits Wg^T, dWg = x^T dlogits, dbias = column sums of dlogits (fp64)."""
    xd, Wd, dl = np.asarray(x, dtype=np.float64), np.asarray(Wg, dtype=np.float64), np.asarray(dlogits, dtype=np.float64)
    return dict(dx=dl @ Wd.T, dWg=xd.T @ dl, dbias=dl.sum(axis=0))


# ---------------------------------------------------------------------------------------------------------------
# Slot assignment (GShard logic kept by the paper, Sec. 2.1; reading R4)
# ---------------------------------------------------------------------------------------------------------------

def bpr_token_order(logits: np.ndarray) -> np.ndarray:
    """Batch prioritized routing (reading R16): tokens in order of decreasing priority, priority = the largest softmax
    probability of the token rounded to fp32; equal priorities keep token order."""
    key = softmax_rows(logits).max(axis=1).astype(np.float32)
    return np.argsort(-key.astype(np.float64), kind="stable")


def slot_locations(idx: np.ndarray, E: int, order: Optional[np.ndarray] = None):
    """loc[t,j] and un-truncated counts[e].

    For each rank j: one-hot mask_j[t,e]; positions = inclusive cumsum over t minus 1; later ranks are offset by
    all arrivals of earlier ranks at that expert.  With `order` (a permutation of the tokens) the tokens arrive in that
    order instead of token order.
    """
    if order is not None:
        loc_o, counts = slot_locations(idx[order], E)
        loc = np.empty_like(loc_o)
        loc[order] = loc_o
        return loc, counts
    T, k = idx.shape
    rows = np.arange(T)
    loc = np.empty((T, k), dtype=np.int64)
    counts = np.zeros(E, dtype=np.int64)
    for j in range(k):
        mask = np.zeros((T, E), dtype=np.int64)
        mask[rows, idx[:, j]] = 1
        pos = np.cumsum(mask, axis=0) - 1 + counts[None, :]
        loc[:, j] = (pos * mask).sum(axis=1)
        counts = counts + mask.sum(axis=0)
    return loc.astype(np.int32), counts.astype(np.int32)


def route(logits: np.ndarray, k: int, C: int, normalize: int, bpr: bool = False) -> Dict[str, np.ndarray]:
    """Gate decisions from fp32 logits: idx, loc, kept, counts, gate_w (fp64), p (fp64); bpr: batch prioritized order."""
    logits = np.asarray(logits, dtype=np.float32)
    E = logits.shape[1]
    idx = topk_experts(logits, k)
    loc, counts = slot_locations(idx, E, bpr_token_order(logits) if bpr else None)
    p = softmax_rows(logits)
    w = gate_weights(p, idx, normalize)
    return dict(idx=idx, loc=loc, kept=(loc < C), counts=counts, gate_w=w, p=p)


def slot_source(idx: np.ndarray, loc: np.ndarray, E: int, C: int) -> np.ndarray:
    """Inverse map slot_src[e,c] = token occupying slot (e,c), or -1 for an unfilled slot."""
    T, k = idx.shape
    src = np.full((E, C), -1, dtype=np.int32)
    for j in range(k):
        t = np.nonzero(loc[:, j] < C)[0]
        src[idx[t, j], loc[t, j]] = t
    return src


# ---------------------------------------------------------------------------------------------------------------
# Dense (definition) encode / decode: Appendix B, dense implementation
# ---------------------------------------------------------------------------------------------------------------

def dense_masks(idx: np.ndarray, loc: np.ndarray, gate_w: np.ndarray, E: int, C: int):
    """dispatch_mask[t,e,c] in {0,1} and combine_w[t,e,c] = gate weight at the same positions."""
    T, k = idx.shape
    D = np.zeros((T, E, C), dtype=np.float64)
    W = np.zeros((T, E, C), dtype=np.float64)
    for j in range(k):
        t = np.nonzero(loc[:, j] < C)[0]
        D[t, idx[t, j], loc[t, j]] += 1.0
        W[t, idx[t, j], loc[t, j]] += gate_w[t, j]
    return D, W


def encode_dense(D: np.ndarray, x: np.ndarray) -> np.ndarray:
    """Z[e,c,m] = sum_t dispatch_mask[t,e,c] x[t,m]   (einsum 'tec,tm->ecm' written as one matmul)."""
    T, E, C = D.shape
    return (D.reshape(T, E * C).T @ np.asarray(x, dtype=np.float64)).reshape(E, C, -1)


def decode_dense(W: np.ndarray, Y: np.ndarray) -> np.ndarray:
    """out[t,m] = sum_{e,c} combine_w[t,e,c] Y[e,c,m]   (einsum 'tec,ecm->tm' written as one matmul)."""
    T, E, C = W.shape
    return W.reshape(T, E * C) @ np.asarray(Y, dtype=np.float64).reshape(E * C, -1)


# ---------------------------------------------------------------------------------------------------------------
# Zero-skipping encode / decode: Appendix B, sparse implementation (same sums, zero terms skipped)
# ---------------------------------------------------------------------------------------------------------------

def encode_sparse(x: np.ndarray, idx: np.ndarray, loc: np.ndarray, E: int, C: int, dtype=np.float64) -> np.ndarray:
    T, k = idx.shape
    Z = np.zeros((E, C, x.shape[1]), dtype=dtype)
    for j in range(k):
        t = np.nonzero(loc[:, j] < C)[0]
        Z[idx[t, j], loc[t, j]] = x[t]
    return Z


def decode_sparse(Y: np.ndarray, idx: np.ndarray, loc: np.ndarray, gate_w: np.ndarray, C: int) -> np.ndarray:
    T, k = idx.shape
    out = np.zeros((T, Y.shape[2]), dtype=np.float64)
    for j in range(k):
        t = np.nonzero(loc[:, j] < C)[0]
        out[t] += gate_w[t, j][:, None] * Y[idx[t, j], loc[t, j]].astype(np.float64)
    return out


# ---------------------------------------------------------------------------------------------------------------
# Backward of encode / decode (Appendix B: differentiable fast encode and decode; reading R14).  The forward maps are
# linear, Z = D^T x and out = W Y, so the backward maps are their transposes; the gate weight enters W linearly.
# ---------------------------------------------------------------------------------------------------------------

def encode_backward_dense(D: np.ndarray, dZ: np.ndarray) -> np.ndarray:
    """dx[t,m] = sum_{e,c} dispatch_mask[t,e,c] dZ[e,c,m]   (einsum 'tec,ecm->tm')."""
    T, E, C = D.shape
    return D.reshape(T, E * C) @ np.asarray(dZ, dtype=np.float64).reshape(E * C, -1)


def decode_backward_dense(W: np.ndarray, d_out: np.ndarray) -> np.ndarray:
    """dY[e,c,m] = sum_t combine_w[t,e,c] d_out[t,m]   (einsum 'tec,tm->ecm')."""
    T, E, C = W.shape
    return (W.reshape(T, E * C).T @ np.asarray(d_out, dtype=np.float64)).reshape(E, C, -1)


def gate_weight_grad(d_out: np.ndarray, Y: np.ndarray, idx: np.ndarray, loc: np.ndarray, C: int) -> np.ndarray:
    """dgate_w[t,j] = sum_m d_out[t,m] Y[idx[t,j], loc[t,j], m] for a kept choice, 0 for a dropped one
    (d out[t,m] / d gate_w[t,j] is the expert-output row of that choice)."""
    T, k = idx.shape
    g = np.zeros((T, k), dtype=np.float64)
    do = np.asarray(d_out, dtype=np.float64)
    for j in range(k):
        t = np.nonzero(loc[:, j] < C)[0]
        g[t, j] = (do[t] * np.asarray(Y[idx[t, j], loc[t, j]], dtype=np.float64)).sum(axis=1)
    return g


def encode_backward_sparse(dZ: np.ndarray, idx: np.ndarray, loc: np.ndarray, C: int) -> np.ndarray:
    """The same sum as encode_backward_dense with the zero terms skipped."""
    T, k = idx.shape
    dx = np.zeros((T, dZ.shape[2]), dtype=np.float64)
    for j in range(k):
        t = np.nonzero(loc[:, j] < C)[0]
        dx[t] += np.asarray(dZ[idx[t, j], loc[t, j]], dtype=np.float64)
    return dx


def decode_backward_sparse(d_out: np.ndarray, idx: np.ndarray, loc: np.ndarray, gate_w: np.ndarray, E: int, C: int) -> np.ndarray:
    """The same sum as decode_backward_dense with the zero terms skipped (one term per filled slot)."""
    T, k = idx.shape
    dY = np.zeros((E, C, d_out.shape[1]), dtype=np.float64)
    for j in range(k):
        t = np.nonzero(loc[:, j] < C)[0]
        dY[idx[t, j], loc[t, j]] = gate_w[t, j][:, None] * np.asarray(d_out[t], dtype=np.float64)
    return dY


# ---------------------------------------------------------------------------------------------------------------
# Expert feed-forward layer (Sec. 2.1: "a feed-forward network layer (fflayer)"; reading R7)
# ---------------------------------------------------------------------------------------------------------------

def activation(h: np.ndarray, act: int) -> np.ndarray:
    if act == ACT_RELU:
        return np.maximum(h, 0.0)
    if act == ACT_GELU:
        return 0.5 * h * (1.0 + _erf(h / math.sqrt(2.0)))
    if act == ACT_SILU:
        return h / (1.0 + np.exp(-h))
    raise ValueError(f"unknown activation {act}")


def ffn_rows(z: np.ndarray, W1e, b1e, W2e, b2e, act: int) -> np.ndarray:
    """One expert on a [rows, M] slab: act(z W1 + b1) W2 + b2 in fp64."""
    h = np.asarray(z, dtype=np.float64) @ np.asarray(W1e, dtype=np.float64)
    if b1e is not None:
        h = h + np.asarray(b1e, dtype=np.float64)[None, :]
    h = activation(h, act)
    y = h @ np.asarray(W2e, dtype=np.float64)
    if b2e is not None:
        y = y + np.asarray(b2e, dtype=np.float64)[None, :]
    return y


def activation_grad(h: np.ndarray, act: int) -> np.ndarray:
    """d act(h) / d h."""
    if act == ACT_RELU:
        return (h > 0.0).astype(np.float64)
    if act == ACT_GELU:                                # d/dh [h Phi(h)] = Phi(h) + h phi(h)
        return 0.5 * (1.0 + _erf(h / math.sqrt(2.0))) + h * np.exp(-0.5 * h * h) / math.sqrt(2.0 * math.pi)
    if act == ACT_SILU:                                # d/dh [h s(h)] = s (1 + h (1 - s))
        sg = 1.0 / (1.0 + np.exp(-h))
        return sg * (1.0 + h * (1.0 - sg))
    raise ValueError(f"unknown activation {act}")


def ffn_rows_backward(z: np.ndarray, W1e, b1e, W2e, dy: np.ndarray, act: int) -> Dict[str, np.ndarray]:
    """Chain rule through one expert on a [rows, M] slab (fp64): gradients of sum(dy * y) with y = ffn_rows(z, ...)."""
    z = np.asarray(z, dtype=np.float64)
    dy = np.asarray(dy, dtype=np.float64)
    W1e, W2e = np.asarray(W1e, dtype=np.float64), np.asarray(W2e, dtype=np.float64)
    pre = z @ W1e
    if b1e is not None:
        pre = pre + np.asarray(b1e, dtype=np.float64)[None, :]
    h = activation(pre, act)
    dh = dy @ W2e.T
    dpre = dh * activation_grad(pre, act)
    return dict(dz=dpre @ W1e.T, dW1=z.T @ dpre, db1=dpre.sum(axis=0), dW2=h.T @ dy, db2=dy.sum(axis=0))


def expert_ffn_backward(Z: np.ndarray, W1, b1, W2, dY: np.ndarray, act: int,
                        rows: Optional[Sequence[int]] = None) -> Dict[str, np.ndarray]:
    """Backward of expert_ffn for every expert; only the first rows[e] rows of an expert exist (others: dZ = 0)."""
    E, C, M = Z.shape
    H = np.asarray(W1[0]).shape[1]
    out = dict(dZ=np.zeros((E, C, M)), dW1=np.zeros((E, M, H)), db1=np.zeros((E, H)), dW2=np.zeros((E, H, M)), db2=np.zeros((E, M)))
    for e in range(E):
        n = C if rows is None else int(min(max(rows[e], 0), C))
        g = ffn_rows_backward(Z[e, :n], W1[e], None if b1 is None else b1[e], W2[e], dY[e, :n], act)
        out["dZ"][e, :n] = g["dz"]
        for name in ("dW1", "db1", "dW2", "db2"):
            out[name][e] = g[name]
    return out


def expert_ffn(Z: np.ndarray, W1, b1, W2, b2, act: int, rows: Optional[Sequence[int]] = None) -> np.ndarray:
    """Y[e] = FFN_e(Z[e]) for every expert, one expert at a time.

    `rows[e]`, if given, limits the work to the first rows[e] slots of expert e (the filled ones); the remaining
    rows of Y are left zero and are never read by decode because their combine weight is zero.
    """
    E, C, M = Z.shape
    Y = np.zeros((E, C, W2.shape[2]), dtype=np.float64)
    for e in range(E):
        r = C if rows is None else int(min(rows[e], C))
        if r > 0:
            Y[e, :r] = ffn_rows(Z[e, :r], W1[e], None if b1 is None else b1[e], W2[e], None if b2 is None else b2[e], act)
    return Y


# ---------------------------------------------------------------------------------------------------------------
# Whole layer
# ---------------------------------------------------------------------------------------------------------------

def moe_layer(x, Wg, gate_bias, W1, b1, W2, b2, k: int, f: float, normalize: int, act: int,
              tier: str = "sparse", logits: Optional[np.ndarray] = None,
              capacity_setting: Optional[float] = None) -> Dict[str, np.ndarray]:
    """gate -> encode -> expert FFN -> decode on one device (Sec. 2.1 with both all-to-alls the identity).

    With `capacity_setting` given, the capacity follows Sec. 4.1's dynamic capacity factor instead of `f`.

    tier = "dense": the literal one-hot-mask contractions (needs a [T,E,C] mask: small inputs only).
    tier = "sparse": the same sums with zero terms skipped; the FFN visits filled slots only.
    """
    T = x.shape[0]
    E = W1.shape[0]
    if logits is None:
        logits = gate_logits(x, Wg, gate_bias)
    if capacity_setting is None:
        C = capacity(T, E, k, f)
    else:                                             # arrivals do not depend on the capacity: count first, then choose C
        C = dynamic_capacity(route(logits, k, 1, normalize)["counts"], T, E, k, capacity_setting)
    r = route(logits, k, C, normalize)
    if tier == "dense":
        D, W = dense_masks(r["idx"], r["loc"], r["gate_w"], E, C)
        Z = encode_dense(D, x)
        Y = expert_ffn(Z, W1, b1, W2, b2, act)
        out = decode_dense(W, Y)
    elif tier == "sparse":
        Z = encode_sparse(x, r["idx"], r["loc"], E, C)
        Y = expert_ffn(Z, W1, b1, W2, b2, act, rows=r["counts"])
        out = decode_sparse(Y, r["idx"], r["loc"], r["gate_w"], C)
    else:
        raise ValueError(tier)
    r.update(C=C, logits=logits, Z=Z, Y=Y, out=out)
    return r


def moe_layer_backward(x, Wg, gate_bias, W1, b1, W2, b2, k: int, f: float, normalize: int, act: int,
                       d_out: np.ndarray) -> Dict[str, np.ndarray]:
    """Backward of moe_layer for a given d loss / d out [T,M] (fp64): the backward maps of decode, the expert layer,
    encode and the gate chained in reverse order, with the routing decisions of the forward held fixed."""
    r = moe_layer(x, Wg, gate_bias, W1, b1, W2, b2, k, f, normalize, act, tier="sparse")
    E, C = W1.shape[0], r["C"]
    idx, loc = r["idx"], r["loc"]
    dY = decode_backward_sparse(d_out, idx, loc, r["gate_w"], E, C)
    dgw = gate_weight_grad(d_out, r["Y"], idx, loc, C)
    rows = np.minimum(r["counts"], C)
    g = expert_ffn_backward(r["Z"], W1, b1, W2, dY, act, rows=rows)
    dlogits = gate_backward(r["logits"], idx, dgw, normalize)
    gb = gate_logits_backward(x, Wg, dlogits)
    return dict(dx=encode_backward_sparse(g["dZ"], idx, loc, C) + gb["dx"], dWg=gb["dWg"], dgate_bias=gb["dbias"],
                dW1=g["dW1"], db1=g["db1"], dW2=g["dW2"], db2=g["db2"], forward=r)


def expert_slabs(x, idx, loc, gate_w, C: int, W1, b1, W2, b2, act: int):
    """Zero-skipping tier streamed one expert at a time (for sizes whose [E,C,M] buffers do not fit in host memory).

    Yields, for e = 0 .. E-1: (e, tokens, w, Z_e, Y_e) with tokens[c] = the token in slot (e, c) for c below the
    expert's fill, w[c] = its gate weight there, Z_e = the dispatched rows x[tokens] (what encode puts into the
    filled rows of slab e; Appendix B) and Y_e = FFN_e(Z_e) in fp64.  Nothing larger than one slab exists at a time.
    """
    E = W1.shape[0]
    tt, jj = np.nonzero(loc < C)                      # kept (token, choice) pairs
    ee, ll = idx[tt, jj], loc[tt, jj]
    order = np.lexsort((ll, ee))                      # by expert, then by slot
    tt, jj, ee, ll = tt[order], jj[order], ee[order], ll[order]
    first = np.searchsorted(ee, np.arange(E + 1))
    for e in range(E):
        a, b = first[e], first[e + 1]
        tokens = tt[a:b]
        assert np.array_equal(ll[a:b], np.arange(b - a)), "kept locations of an expert must be 0 .. fill-1, each once"
        Ze = np.asarray(x[tokens], dtype=np.float64)
        Ye = ffn_rows(Ze, W1[e], None if b1 is None else b1[e], W2[e], None if b2 is None else b2[e], act) \
            if b > a else np.zeros((0, W2.shape[2]))
        yield e, tokens, np.asarray(gate_w[tokens, jj[a:b]], dtype=np.float64), Ze, Ye


def moe_layer_streamed(x, Wg, gate_bias, W1, b1, W2, b2, k: int, f: float, normalize: int, act: int,
                       logits: Optional[np.ndarray] = None, on_expert=None) -> Dict[str, np.ndarray]:
    """moe_layer's result without any [E,C,M] buffer: the combine sum  out[t] = sum_{e,c} combine_w[t,e,c] Y[e,c]  of
    the dense definition (Appendix B) visited expert by expert, slots ascending, zero terms skipped.

    `on_expert(e, tokens, w, Z_e, Y_e)`, if given, sees every expert's filled slab as it is produced (the caller can
    compare it with the device's slab and drop it).  Returns routing, logits, C and out (no Z, no Y).
    """
    T, E = x.shape[0], W1.shape[0]
    if logits is None:
        logits = gate_logits(x, Wg, gate_bias)
    C = capacity(T, E, k, f)
    r = route(logits, k, C, normalize)
    out = np.zeros((T, W2.shape[2]), dtype=np.float64)
    for e, tokens, w, Ze, Ye in expert_slabs(x, r["idx"], r["loc"], r["gate_w"], C, W1, b1, W2, b2, act):
        if on_expert is not None:
            on_expert(e, tokens, w, Ze, Ye)
        out[tokens] += w[:, None] * Ye                # a token sits in at most one slot of an expert: no index repeats
    r.update(C=C, logits=logits, out=out)
    return r


def token_outputs_direct(tokens: Sequence[int], x, idx, loc, gate_w, C: int, W1, b1, W2, b2, act: int) -> np.ndarray:
    """out[t,:] = sum over kept choices j of gate_w[t,j] * FFN_{idx[t,j]}(x[t,:]), with no [E,C,M] buffers.

    Used for sampled rows at sizes where the buffered oracle would not fit, and as a cross-check of it.
    """
    tokens = np.asarray(tokens, dtype=np.int64)
    out = np.zeros((len(tokens), W2.shape[2]), dtype=np.float64)
    k = idx.shape[1]
    for j in range(k):
        sel = np.nonzero(loc[tokens, j] < C)[0]
        if sel.size == 0:
            continue
        experts = idx[tokens[sel], j]
        for e in np.unique(experts):
            s = sel[experts == e]
            y = ffn_rows(x[tokens[s]], W1[e], None if b1 is None else b1[e], W2[e], None if b2 is None else b2[e], act)
            out[s] += gate_w[tokens[s], j][:, None] * y
    return out


# ---------------------------------------------------------------------------------------------------------------
# Brute force, independent of everything above except `activation` (tiny inputs only)
# ---------------------------------------------------------------------------------------------------------------

def brute_force_route(logits: np.ndarray, k: int, C: int, order: Optional[Sequence[int]] = None):
    """Sequential arrival simulation with plain Python loops: for each rank, for each token (in `order` if given), take
    the next slot."""
    T, E = logits.shape
    order = list(range(T)) if order is None else [int(t) for t in order]
    choice = [[-1] * k for _ in range(T)]
    for t in range(T):
        taken = set()
        for j in range(k):
            best = None
            for e in range(E):
                if e in taken:
                    continue
                if best is None or float(np.float32(logits[t, e])) > float(np.float32(logits[t, best])):
                    best = e
            taken.add(best)
            choice[t][j] = best
    arrivals = [0] * E
    loc = [[-1] * k for _ in range(T)]
    for j in range(k):
        for t in order:
            e = choice[t][j]
            loc[t][j] = arrivals[e]
            arrivals[e] += 1
    idx = np.array(choice, dtype=np.int32)
    loc = np.array(loc, dtype=np.int32)
    return idx, loc, loc < C, np.array(arrivals, dtype=np.int32)


def brute_force_layer(x, Wg, gate_bias, W1, b1, W2, b2, k, f, normalize, act) -> np.ndarray:
    """Per token, per kept choice: run the chosen expert on the token's row and add it, scaled by its gate weight."""
    T, M = x.shape
    E = W1.shape[0]
    C = capacity(T, E, k, f)
    logits = np.zeros((T, E), dtype=np.float32)
    for t in range(T):
        for e in range(E):
            s = 0.0
            for m in range(M):
                s += float(x[t, m]) * float(Wg[m, e])
            if gate_bias is not None:
                s += float(gate_bias[e])
            logits[t, e] = np.float32(s)
    idx, loc, kept, _ = brute_force_route(logits, k, C)
    out = np.zeros((T, W2.shape[2]), dtype=np.float64)
    for t in range(T):
        z = [float(v) for v in logits[t]]
        mx = max(z)
        ex = [math.exp(v - mx) for v in z]
        den = sum(ex)
        p = [v / den for v in ex]
        wsum = sum(p[idx[t, j]] for j in range(k))
        for j in range(k):
            if not kept[t, j]:
                continue
            e = int(idx[t, j])
            w = p[e] / wsum if normalize else p[e]
            h = np.array([sum(float(x[t, m]) * float(W1[e, m, n]) for m in range(M)) + (0.0 if b1 is None else float(b1[e, n]))
                          for n in range(W1.shape[2])])
            h = activation(h, act)
            y = np.array([sum(h[n] * float(W2[e, n, m]) for n in range(W2.shape[1])) + (0.0 if b2 is None else float(b2[e, m]))
                          for m in range(W2.shape[2])])
            out[t] += w * y
    return out
