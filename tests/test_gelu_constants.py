"""The HIP kernels' GeLU evaluates erfc(|z| / sqrt 2) as 2^P(|z|) with fitted coefficients
(csrc/common.h).  This host-side test reads those constants from the source and re-evaluates the
formula in fp32 against scipy's erf: the approximation error the kernel comments state must hold,
the polynomial must stay negative (2^P <= 1) and fall to -inf far out, and the tail must keep
its relative accuracy (no 1 + erf cancellation)."""
import os
import re

import numpy as np
from scipy.special import erf

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def coefficients():
    text = open(os.path.join(ROOT, "paper_2209_02341_amd", "csrc", "common.h")).read()
    body = re.search(r"kGeluErfcPoly\[7\]\s*=\s*\{(.*?)\}", text, flags=re.S).group(1)
    vals = [np.float32(v.strip().rstrip("f")) for v in body.split(",")]
    assert len(vals) == 7
    return vals


def gelu_kernel_formula(z32):
    c = coefficients()
    a = np.abs(z32)
    p = np.full_like(a, c[6])
    with np.errstate(over="ignore"):   # far out P runs to -inf on purpose
        for k in range(5, -1, -1):
            p = p * a + c[k]
        pa = p * a
        e = np.exp2(pa)
        return np.maximum(z32, np.float32(0)) - np.float32(0.5) * a * e, pa


def test_gelu_polynomial_matches_erf_form():
    z = np.linspace(-12, 12, 600001).astype(np.float32)
    got, p = gelu_kernel_formula(z)
    z64 = z.astype(np.float64)
    ref = 0.5 * z64 * (1.0 + erf(z64 / np.sqrt(2.0)))
    err = np.abs(got.astype(np.float64) - ref)
    # approximation error 1.3e-7 plus half an fp32 ulp of the result
    assert np.all(err <= 1.3e-7 + 2.0 ** -24 * np.abs(ref))
    assert np.all(p <= 0)
    tail = (z < -0.5) & (z > -6)
    assert (err[tail] / np.abs(ref[tail])).max() < 0.06


def test_gelu_polynomial_far_out():
    z = np.array([30, -30, 1e3, -1e3, 6e4, -6e4, 1e20, -1e20, 0.0, 1e-8, -1e-8], dtype=np.float32)
    got, p = gelu_kernel_formula(z)
    want = np.array([30, 0, 1e3, 0, 6e4, 0, 1e20, 0, 0, 5e-9, -5e-9], dtype=np.float32)
    assert np.allclose(got, want, rtol=1e-6, atol=0)
    assert np.all(np.isfinite(got))
    zz = np.logspace(0, 38, 4000).astype(np.float32)
    _, pp = gelu_kernel_formula(zz)
    assert np.all(pp < 0) and not np.any(np.isnan(pp))
