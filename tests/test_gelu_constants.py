"""Host-side check of the constants the bf16 FFN epilogue uses for GELU.

The kernel source holds seven float coefficients of a polynomial P with Phi(-a) = exp2(P(a)); this test
reads them out of the source text, evaluates the kernel's formula step by step in float32 with numpy,
and compares with the erf definition of GELU (scipy), so a mistyped coefficient or a wrong clamp fails
here, on the CPU, before any GPU run.  It also checks that the committed fit script still reproduces
the constants.
"""
import os
import re

import numpy as np
from scipy.special import erf

from paper_2411_16786_amd import gelu_fit

HEADER = os.path.join(os.path.dirname(__file__), "..", "paper_2411_16786_amd", "csrc", "ffn_mfma.hpp")


def _kernel_coefficients():
    text = open(HEADER).read()
    body = text[text.index("float gelu_erf_fast(float u)"):]
    body = body[:body.index("}")]
    hexes = re.findall(r"(-?0x1\.[0-9a-f]+p[+-]\d+)f", body)
    assert len(hexes) == 7, hexes
    # Horner order in the source: highest degree first
    coef = [float.fromhex(h) for h in hexes][::-1]
    clamp = re.search(r"fminf\(fabsf\(u\), ([0-9.]+)f\)", body)
    assert clamp and float(clamp.group(1)) == gelu_fit.A_MAX
    return np.array(coef, dtype=np.float32)


def test_kernel_gelu_formula_matches_erf_definition():
    coef = _kernel_coefficients()
    u = np.linspace(-12.0, 12.0, 480001)
    got = gelu_fit.gelu_float32(u, coef).astype(np.float64)
    exact = 0.5 * u * (1.0 + erf(u / np.sqrt(2.0)))
    err = np.abs(got - exact)
    # float32 rounding of the result itself is 2.4e-7 at |u| = 4; bf16 rounding, applied next, is 2^-9 relative
    assert err.max() < 1e-6
    big = np.abs(exact) > 1e-3
    assert (err[big] / np.abs(exact[big])).max() < 1e-4      # bf16 rounding is 2e-3 relative


def test_fit_script_reproduces_kernel_constants():
    coef = _kernel_coefficients()
    refit = gelu_fit.fit()
    assert refit.shape == coef.shape
    np.testing.assert_allclose(refit, coef, rtol=2e-6, atol=0)
