"""Derives the polynomial in gelu_to_half_bits (common.h) and reports its error.  Not part of the build.

erfc(z) = t exp(-z^2 + g(t)) with t = 1 / (1 + z / 2): g(t) = ln(exp(z^2) erfc(z) / t) is smooth on (0, 1], and a
Chebyshev fit of degree 8 on the t range that |x| <= 13.5 maps to (z = |x| / sqrt 2) is converted to a power
series.  The error is measured on the kernel's own arithmetic: float32, Horner with fused multiply-adds (emulated
here as a float64 product and sum rounded once to float32).
Run: python gelu_coefficients.py"""
import numpy as np
from scipy.special import erfc, erfcx   # erfcx(z) = exp(z^2) erfc(z)

DEGREE = 8
X_MAX = 13.5


def fit():
    t_min = 1.0 / (1.0 + 0.5 * X_MAX / np.sqrt(2.0))
    k = np.arange(4000)
    u = np.cos(np.pi * (k + 0.5) / 4000)                                  # Chebyshev nodes on [-1, 1]
    t = 0.5 * (1 + t_min) + 0.5 * (1 - t_min) * u
    z = 2.0 * (1.0 / t - 1.0)
    cheb = np.polynomial.chebyshev.chebfit(u, np.log(erfcx(z) / t), DEGREE)
    in_u = np.polynomial.Polynomial(np.polynomial.chebyshev.cheb2poly(cheb))
    in_t = in_u(np.polynomial.Polynomial([-(1 + t_min) / (1 - t_min), 2 / (1 - t_min)]))
    return in_t.coef


def error(coef):
    f = np.float32
    x = np.linspace(0.0, X_MAX, 200001)
    def fma(a, b, c):
        return (a.astype(np.float64) * np.asarray(b, np.float64) + np.asarray(c, np.float64)).astype(f)

    z = (x.astype(f) * f(0.70710678118654752)).astype(f)
    t = (f(1) / fma(z, f(0.5), f(1))).astype(f)
    g = np.full_like(t, f(coef[-1]))
    for c in coef[-2::-1]:
        g = fma(g, t, f(c))
    arg = fma(-z, z, g)
    got = (t * np.exp(arg.astype(np.float64))).astype(f)
    ref = erfc(x / np.sqrt(2.0))
    rel = np.abs(got - ref) / ref
    return rel[x < 5.5].max(), rel.max()


if __name__ == "__main__":
    c = fit()
    print("coefficients, constant term first:")
    print(", ".join("%.9ef" % v for v in c))
    near, far = error(c)
    print("relative error of erfc in float32: %.2e for |x| < 5.5, %.2e up to %.1f" % (near, far, X_MAX))
