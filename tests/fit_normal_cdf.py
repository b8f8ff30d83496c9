"""Derives the constants of s24_normal() in paper_2404_01847_amd/csrc/s24_common.h (the GELU kernels' normal CDF);
tests/test_gelu_constants.py refits them with fit() and checks the header against the result.

For s >= 0 the lower tail is written Phi(-s) = exp(-s^2/2) * Q(t) with t = 1 / (1 + P s): Q is smooth on (0, 1],
vanishes linearly at t = 0 (the Mills ratio) and equals 1/2 at t = 1, so Q(t) = t * poly(t) fits well, and because
the exponential is factored out the RELATIVE accuracy of the tail survives far from the origin.  The fit is a
weighted least-squares fit of Q(t)/t in a Chebyshev basis with Lawson reweighting towards the minimax solution,
against scipy's scaled complementary error function; the script then evaluates Phi, GELU and GELU' in emulated fp32
with the rounded coefficients against fp64 references and prints the errors and the constants.

    python tests/fit_normal_cdf.py
"""
import numpy as np
from numpy.polynomial import Polynomial
from numpy.polynomial import chebyshev as C
from scipy.special import erfcx, ndtr

P, DEGREE = 0.375, 9


def q_exact(s):
    return 0.5 * erfcx(s / np.sqrt(2.0))          # Phi(-s) * exp(s^2 / 2)


def fit(p=P, deg=DEGREE, n=4000, sweeps=60):
    k = np.arange(n)
    t = 0.5 * (1 - np.cos(np.pi * (k + 0.5) / n))
    y = q_exact((1.0 / t - 1.0) / p) / t
    V = C.chebvander(2 * t - 1, deg - 1)
    lawson = np.ones(n)
    for _ in range(sweeps):
        c = np.linalg.lstsq(V * (lawson / y)[:, None], lawson, rcond=None)[0]
        r = np.abs(V @ c / y - 1.0)
        lawson = lawson * np.sqrt(r / r.max() + 1e-3)
        lawson /= lawson.max()
    poly, power, x_of_t = Polynomial([0.0]), Polynomial([1.0]), Polynomial([-1.0, 2.0])
    for a in C.cheb2poly(c):
        poly, power = poly + a * power, power * x_of_t
    return poly.coef, np.abs(V @ c / y - 1.0).max()


def main():
    coef, err = fit()
    c32 = coef.astype(np.float32)
    print(f"P = {P}, degree {DEGREE}: relative error of the fit {err:.3e}")
    print("coefficients of t^1 .. t^%d:" % DEGREE, ", ".join(f"{v:.9e}f" for v in c32))
    f32 = np.float32
    x = np.linspace(-9, 9, 2000001).astype(f32)
    t = (f32(1) / (f32(1) + f32(P) * np.abs(x))).astype(f32)
    q = np.zeros_like(t) + c32[-1]
    for a in c32[-2::-1]:
        q = (q * t + a).astype(f32)
    e = np.exp2((f32(-0.72134752) * x * x).astype(f32)).astype(f32)
    tail = (e * (q * t).astype(f32)).astype(f32)
    cdf = np.where(x < 0, tail, (f32(1) - tail).astype(f32))
    xd = x.astype(np.float64)
    ref = ndtr(xd)
    for name, got, want in (("Phi", cdf, ref), ("GELU", x * cdf, xd * ref),
                            ("GELU'", cdf + x * (e * f32(0.3989422804)), ref + xd * np.exp(-0.5 * xd * xd) / np.sqrt(2 * np.pi))):
        d = np.abs(got.astype(np.float64) - want)
        print(f"{name:6s} max abs error {d.max():.3e}")
    print(f"Phi    max relative error {np.abs(cdf / ref - 1).max():.3e} (the lower tail keeps its relative accuracy)")


if __name__ == "__main__":
    main()
