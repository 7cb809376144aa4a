"""Host-side checks of closed-form approximations that the HIP kernels use (no GPU needed).

The decode-step kernels evaluate erf by formula 7.1.26 of Abramowitz & Stegun instead of calling the library
routine.  The coefficients are read out of the kernel source, the formula is evaluated in fp32 exactly as the
device code does, and the result is compared with scipy's erf: the GELU built on it must stay three orders of
magnitude below the fp16 rounding of its output (half an ulp of fp16 at |y| = 1 is 4.9e-4).
"""
import os
import re

import numpy as np
from scipy.special import erf

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _coefficients():
    src = open(os.path.join(ROOT, "paper_2407_04991_amd", "csrc", "common.h")).read()
    body = src[src.index("float erf_as(float x)"):]
    body = body[:body.index("}")]
    p = float(re.search(r"1\.0f \+ ([0-9.]+)f \* ax", body).group(1))
    poly = re.search(r"poly = \(\(\(\(([0-9.]+)f \* t - ([0-9.]+)f\) \* t \+ ([0-9.]+)f\) \* t - ([0-9.]+)f\) \* t \+ ([0-9.]+)f\) \* t", body)
    a5, a4, a3, a2, a1 = (float(g) for g in poly.groups())
    return p, (a1, -a2, a3, -a4, a5)


def _erf_as_fp32(x, p, a):
    f = np.float32
    ax = np.abs(x).astype(f)
    t = (f(1.0) / (f(1.0) + f(p) * ax)).astype(f)
    poly = f(a[4])
    for c in (a[3], a[2], a[1], a[0]):
        poly = (poly * t + f(c)).astype(f)
    poly = (poly * t).astype(f)
    return np.copysign((f(1.0) - poly * np.exp(-(ax * ax)).astype(f)).astype(f), x)


def test_coefficients_are_the_published_ones():
    p, a = _coefficients()
    assert p == 0.3275911
    assert a == (0.254829592, -0.284496736, 1.421413741, -1.453152027, 1.061405429)


def test_erf_formula_error_bound_in_fp32():
    p, a = _coefficients()
    x = np.linspace(-8.0, 8.0, 2_000_001).astype(np.float32)
    err = np.abs(_erf_as_fp32(x, p, a).astype(np.float64) - erf(x.astype(np.float64)))
    assert err.max() < 7e-7, err.max()


def test_gelu_on_the_formula_is_far_below_fp16_rounding():
    p, a = _coefficients()
    x = np.linspace(-12.0, 12.0, 2_000_001).astype(np.float32)
    s = np.float32(0.70710678118654752440)
    g_fast = (x * np.float32(0.5) * (np.float32(1.0) + _erf_as_fp32((x * s).astype(np.float32), p, a))).astype(np.float64)
    xd = x.astype(np.float64)
    g_ref = xd * 0.5 * (1.0 + erf(xd / np.sqrt(2.0)))
    err = np.abs(g_fast - g_ref)
    assert err.max() < 6e-7, err.max()
    # fp16 spacing at |gelu| ~ 1 is 9.8e-4, at 1e-2 it is 7.6e-6: the approximation error is below both
    assert err.max() < 7.6e-6 / 10
