#!/usr/bin/env python3
"""Derives the polynomial of the bf16 GEMM epilogue's GELU.

gelu(v) = v * Phi(v) with Phi(-y) = erfc(y / sqrt 2) / 2 for y = |v| >= 0.  The epilogue evaluates
    e = 2 ** -P(y),  P(y) = y (c1 + y (c2 + y (c3 + y (c4 + y c5)))),   Phi(v) = 1 - e/2 (v >= 0), e/2 (v < 0),
one exponential and no division.  P is a weighted least-squares fit of -log2 erfc(y / sqrt 2) on [0, 8] whose weights
are iterated towards the minimax of the error it causes in gelu itself (|v| * e/2 * ln 2 * |dP|); past 8 the leading
coefficient keeps P growing, so e underflows to 0 as it should.  Run it to print the coefficients and the resulting
maximum absolute error of gelu in fp32 evaluation (5.7e-7, three orders below bf16 resolution near 1).
"""
import numpy as np
from scipy.special import erf, erfc

DEGREE = 5


def fit():
    y = np.linspace(0.0, 8.0, 200001)
    g = -np.log2(erfc(y / np.sqrt(2.0)))
    sens = y * 0.5 * erfc(y / np.sqrt(2.0)) * np.log(2.0)          # d gelu / d P
    A = np.stack([y ** k for k in range(1, DEGREE + 1)], axis=1)
    w = sens + 1e-12
    for _ in range(30):
        c, *_ = np.linalg.lstsq(A * w[:, None], g * w, rcond=None)
        err = np.abs((A @ c - g) * sens)
        w = w * (1.0 + 3.0 * err / err.max())
    return c.astype(np.float32)


def max_gelu_error(c32):
    y = np.linspace(0.0, 12.0, 300001).astype(np.float32)
    P = np.zeros_like(y)
    for k in range(DEGREE - 1, -1, -1):
        P = (P + c32[k]) * y                                       # fp32 Horner, as the kernel does
    e = np.exp2(-P.astype(np.float64))
    worst = 0.0
    for sign in (1.0, -1.0):
        v = sign * y.astype(np.float64)
        phi = np.where(v >= 0, 1.0 - 0.5 * e, 0.5 * e)
        worst = max(worst, float(np.abs(v * phi - 0.5 * v * (1.0 + erf(v / np.sqrt(2.0)))).max()))
    return worst


if __name__ == "__main__":
    c = fit()
    print("coefficients c1..c5:", ", ".join(f"{float(x):.9e}f" for x in c))
    print("max |gelu error| on [-12, 12]: %.3e" % max_gelu_error(c))
