"""Coefficients of the GELU used in the bf16 FFN epilogue (csrc/ffn_mfma.hpp, gelu_erf_fast).

The expert FFN applies the exact (erf) GELU, gelu(u) = u Phi(u).  The kernel evaluates it as

    gelu(u) = max(u, 0) - a Phi(-a),      a = min(|u|, 6),     Phi(-a) = exp2(P(a)),

with P a degree-6 polynomial fitted to log2 Phi(-a) on [0, 6].  The fit minimises the largest
weighted error, the weight being a Phi(-a) (the factor that turns an error of P into an absolute
error of the result) with a floor proportional to Phi(-a) (so that the relative error stays small
where the result itself is small).  Running this file prints the coefficients as C hex floats, lowest
degree first, and the largest error of the formula in float arithmetic against the erf definition.

This module serves the HIP path only; the test oracle does not use it.
"""
import numpy as np
from numpy.polynomial import chebyshev as cheb
from scipy.special import erf, erfc

A_MAX = 6.0
DEGREE = 6


def fit(degree=DEGREE, a_max=A_MAX, samples=20001, sweeps=200):
    """Monomial coefficients (lowest degree first, float32) of P(a) ~ log2 Phi(-a) on [0, a_max]."""
    a = np.linspace(0.0, a_max, samples)
    phi = 0.5 * erfc(a / np.sqrt(2.0))
    target = np.log2(phi)
    weight = np.maximum(a * phi, 0.02 * phi)
    w = weight.copy()
    x = 2.0 * a / a_max - 1.0
    for _ in range(sweeps):                       # reweighted least squares -> near-minimax
        coef = cheb.chebfit(x, target, degree, w=w)
        err = np.abs((cheb.chebval(x, coef) - target) * weight)
        w = w * np.sqrt(1.0 + 2.0 * err / err.max())
        w /= w.max()
    # Chebyshev series in x = 2a/a_max - 1  ->  power series in a
    powers_of_x = cheb.cheb2poly(coef)
    lin = np.polynomial.Polynomial([-1.0, 2.0 / a_max])
    p = np.polynomial.Polynomial([0.0])
    for k, ck in enumerate(powers_of_x):
        p = p + ck * lin ** k
    return p.coef.astype(np.float32)


def gelu_float32(u, coef):
    """The kernel's formula, evaluated step by step in float32."""
    u = np.asarray(u, dtype=np.float32)
    a = np.minimum(np.abs(u), np.float32(A_MAX))
    p = np.full_like(a, coef[-1])
    for c in coef[-2::-1]:
        p = (p * a + np.float32(c)).astype(np.float32)
    tail = np.exp2(p).astype(np.float32)
    return (np.maximum(u, np.float32(0.0)) - a * tail).astype(np.float32)


def gelu_exact(u):
    u = np.asarray(u, dtype=np.float64)
    return 0.5 * u * (1.0 + erf(u / np.sqrt(2.0)))


if __name__ == "__main__":
    c = fit()
    print("coefficients, lowest degree first:")
    for ck in c:
        print("   ", float(ck).hex(), float(ck))
    u = np.linspace(-10.0, 10.0, 800001)
    d = np.abs(gelu_float32(u, c).astype(np.float64) - gelu_exact(u))
    print("largest |formula - exact| in float32 on [-10, 10]: %.3e at u = %.3f" % (d.max(), u[d.argmax()]))
