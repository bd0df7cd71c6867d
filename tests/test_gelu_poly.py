"""The bf16 GEMM epilogue's GELU is v * Phi(v) with Phi from one exponential of a fitted polynomial, and the epilogue
of the backward's dH product uses gelu'(v) = Phi(v) + v phi(v) with the same Phi.  These host-side tests read the
coefficients out of the kernel source and check both formulas, evaluated in fp32 as the kernel does, against the exact
erf forms (the oracle's activation and its derivative) over the whole range that matters and far beyond it."""
import os
import re

import numpy as np

from oracle import moe_oracle as O

SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2206_03382_amd", "csrc", "ffn_mfma.hip")


def kernel_coefficients():
    text = open(SRC).read()
    vals = []
    for i in range(1, 6):
        m = re.search(r"kGeluC%d\s*=\s*([-+0-9.eE]+)f" % i, text)
        assert m, f"kGeluC{i} not found in {SRC}"
        vals.append(np.float32(m.group(1)))
    return vals


def kernel_phi_minus_half(v32):
    c = kernel_coefficients()
    y = np.abs(v32)
    p = np.float32(c[4]) * y + c[3]
    for k in (2, 1, 0):
        p = (p * y + c[k]).astype(np.float32)
    with np.errstate(over="ignore", under="ignore"):
        e = np.exp2(-(p * y).astype(np.float32).astype(np.float64)).astype(np.float32)
    return np.copysign((np.float32(0.5) - np.float32(0.5) * e).astype(np.float32), v32)


def kernel_gelu(v32):
    return (v32 * (np.float32(0.5) + kernel_phi_minus_half(v32))).astype(np.float32)


def kernel_constant(name):
    m = re.search(r"%s\s*=\s*([-+0-9.eE]+)f" % name, open(SRC).read())
    assert m, f"{name} not found in {SRC}"
    return np.float32(m.group(1))


def kernel_gelu_grad(v32):
    with np.errstate(over="ignore", under="ignore"):
        arg = (-kernel_constant("kHalfLog2e") * v32 * v32).astype(np.float32)
        dens = (np.exp2(arg.astype(np.float64)).astype(np.float32) * kernel_constant("kInvSqrt2Pi")).astype(np.float32)
        return (v32 * dens + (np.float32(0.5) + kernel_phi_minus_half(v32))).astype(np.float32)


def test_gelu_polynomial_matches_erf_form():
    v = np.concatenate([np.linspace(-12, 12, 480001), np.array([-0.0, 0.0, 1e-30, -1e-30, 50.0, -50.0, 1e4, -1e4, 1e30, -1e30])])
    v32 = v.astype(np.float32)
    ref = O.activation(v32.astype(np.float64), O.ACT_GELU)
    got = kernel_gelu(v32).astype(np.float64)
    err = np.abs(got - ref)
    tol = 1e-6 + 2e-7 * np.abs(ref)                                # fp32 rounding of the final product scales with |v|
    assert np.all(err <= tol), (float(err.max()), float(v32[np.argmax(err - tol)]))
    assert np.signbit(kernel_gelu(np.array([-0.0], np.float32))[0])


def test_gelu_derivative_matches_erf_form():
    v = np.concatenate([np.linspace(-12, 12, 480001), np.array([-0.0, 0.0, 1e-30, -1e-30, 50.0, -50.0, 1e4, -1e4, 1e18, -1e18])])
    v32 = v.astype(np.float32)
    ref = O.activation_grad(v32.astype(np.float64), O.ACT_GELU)
    got = kernel_gelu_grad(v32).astype(np.float64)
    err = np.abs(got - ref)
    assert np.all(err <= 5e-6), (float(err.max()), float(v32[np.argmax(err)]))
