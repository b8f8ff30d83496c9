"""CPU pin of the GELU kernels' normal-CDF approximation (s24_normal() in csrc/s24_common.h).

The nine polynomial coefficients, the 0.375 of the rational argument and the two scale constants are read from the
header's text and evaluated in emulated fp32, operation by operation as the device function does, against math.erf /
math.exp in fp64 (the erf form of GELU, Sec. 5.2).  The hardware's exp2 and reciprocal are accurate to about one unit in
the last place; the emulation rounds the exact result, so the bounds asserted here leave that much room."""
import math
import os
import re

import numpy as np
import pytest

HEADER = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))),
                      "paper_2404_01847_amd", "csrc", "s24_common.h")
f32 = np.float32


def header_constants():
    src = open(HEADER).read()
    body = src[src.index("void s24_normal(float x"):]
    body = body[:body.index("\n}\n")]
    p = float(re.search(r"fmaf\(([0-9.e+-]+)f, fabsf\(x\), 1\.0f\)", body).group(1))
    lead = float(re.search(r"float q = ([0-9.e+-]+)f;", body).group(1))
    rest = [float(v) for v in re.findall(r"q = fmaf\(q, t, ([0-9.e+-]+)f\);", body)]
    k = float(re.search(r"exp2f\(([0-9.e+-]+)f \* x \* x\)", body).group(1))
    slope = float(re.search(r"fmaf\(x, e \* ([0-9.e+-]+)f, cdf\)", src).group(1))
    return p, [lead] + rest, k, slope


def fma32(a, b, c):
    # products of two fp32 numbers are exact in fp64; the sum then carries a relative 2^-53 before the one rounding
    return (a.astype(np.float64) * b.astype(np.float64) + np.float64(c)).astype(f32)


def normal32(x):
    """s24_normal() step by step in fp32: returns (cdf, e)."""
    p, coef, k, _ = header_constants()
    t = (1.0 / fma32(np.full_like(x, f32(p)), np.abs(x), f32(1.0)).astype(np.float64)).astype(f32)
    q = np.full_like(x, f32(coef[0]))
    for c in coef[1:]:
        q = fma32(q, t, f32(c))
    arg = ((f32(k) * x).astype(f32) * x).astype(f32)
    e = np.exp2(arg.astype(np.float64)).astype(f32)
    tail = (e * (q * t).astype(f32)).astype(f32)
    return np.where(x < 0, tail, (f32(1.0) - tail).astype(f32)), e


def test_header_holds_nine_coefficients_and_the_right_scales():
    p, coef, k, slope = header_constants()
    assert p == 0.375 and len(coef) == 9
    assert abs(k + 0.5 / math.log(2.0)) < 1e-7            # exp(-x^2/2) = 2^(-x^2 / (2 ln 2))
    assert abs(slope - 1.0 / math.sqrt(2.0 * math.pi)) < 1e-9


def test_normal_cdf_gelu_and_slope_against_erf():
    x = np.concatenate([np.linspace(-12.0, 12.0, 480001), [0.0, -0.0, 1e-8, -1e-8, 1e-3, -1e-3]]).astype(f32)
    cdf, e = normal32(x)
    _, _, _, slope = header_constants()
    xd = x.astype(np.float64)
    phi = np.array([0.5 * (1.0 + math.erf(v / math.sqrt(2.0))) for v in xd])
    phi_low = np.array([0.5 * math.erfc(-v / math.sqrt(2.0)) for v in xd])     # accurate in the lower tail
    phi = np.where(xd < 0, phi_low, phi)
    dens = np.exp(-0.5 * xd * xd) / math.sqrt(2.0 * math.pi)
    assert np.abs(cdf.astype(np.float64) - phi).max() < 4e-7
    gelu = (x * cdf).astype(f32).astype(np.float64)
    assert (np.abs(gelu - xd * phi) / np.maximum(1.0, np.abs(xd))).max() < 4e-7
    gslope = fma32(x, (e * f32(slope)).astype(f32), cdf).astype(np.float64)
    assert np.abs(gslope - (phi + xd * dens)).max() < 4e-7
    # the lower tail keeps its RELATIVE accuracy (the exponential is a factor): down to where fp32 runs out of range
    low = (xd <= 0) & (xd >= -12.0)
    assert np.abs(cdf[low].astype(np.float64) / phi[low] - 1.0).max() < 1e-5
    # exact anchors
    zero = normal32(np.array([0.0], dtype=f32))[0][0]
    assert abs(float(zero) - 0.5) < 2e-7
    assert float((x * cdf)[np.where(x == 0)[0][0]]) == 0.0
    # monotone within rounding, and inside [0, 1]
    order = np.argsort(x[:480001], kind="stable")
    assert (np.diff(cdf[:480001][order].astype(np.float64)) > -3e-7).all()
    assert cdf.min() >= 0.0 and cdf.max() <= 1.0


def test_constants_are_what_the_fit_produces():
    pytest.importorskip("scipy")
    import fit_normal_cdf as fit
    coef, err = fit.fit()
    _, header, _, _ = header_constants()
    assert err < 5e-6
    # the header lists the polynomial from the highest power down; the fit returns ascending powers of Q(t)/t
    np.testing.assert_allclose(np.array(header[::-1]), coef.astype(f32), rtol=0, atol=2e-7)
