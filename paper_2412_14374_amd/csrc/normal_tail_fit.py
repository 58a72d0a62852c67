"""Writes the coefficients of normal_cdf_fit (device_utils.h) and the error of its fp32
evaluation.  Run: python paper_2412_14374_amd/csrc/normal_tail_fit.py

The upper tail of the standard normal, 1 - Phi(u) = erfc(u / sqrt 2) / 2, is written as
2^(u Q(u)) / 2; Q(u) = log2(erfc(u / sqrt 2)) / u is smooth on [0, 5.7] (Q(0) =
-sqrt(2 / pi) / ln 2) and is fitted there by a degree-8 polynomial, least squares at 4000
Chebyshev nodes.  The evaluation below repeats the kernel's steps in numpy float32 (Horner
with fused multiply-adds replaced by rounded multiply and add, which is no more accurate)."""
import numpy as np
from numpy.polynomial import chebyshev, polynomial
from scipy.special import erf, erfc

U_MAX, DEGREE, NODES = 5.7, 8, 4000


def fit():
    k = np.arange(NODES) + 0.5
    u = (np.cos(np.pi * k / NODES) + 1.0) * U_MAX / 2
    q = np.log2(erfc(u / np.sqrt(2.0))) / u
    c = chebyshev.Chebyshev.fit(u, q, DEGREE, domain=[0, U_MAX])
    return c.convert(kind=polynomial.Polynomial).convert(domain=[-1, 1]).coef    # powers of u, ascending


def normal_cdf_f32(coef, h):
    f = np.float32
    u = np.minimum(np.abs(h), f(U_MAX)).astype(f)
    q = np.full_like(u, f(coef[-1]))
    for c in coef[-2::-1]:
        q = (q * u + f(c)).astype(f)
    tail2 = np.exp2((q * u).astype(f)).astype(f)
    return (f(0.5) + np.copysign((f(0.5) - f(0.5) * tail2).astype(f), h)).astype(f)


if __name__ == "__main__":
    coef = fit()
    print("coefficients of u^0 .. u^%d:" % DEGREE)
    print(", ".join("%.9ef" % np.float32(c) for c in coef))
    h = np.linspace(-8, 8, 2000001).astype(np.float32)
    exact = 0.5 * (1 + erf(h.astype(np.float64) / np.sqrt(2.0)))
    phi = normal_cdf_f32(coef, h)
    print("max |Phi error| on [-8, 8]:   %.2e" % np.abs(phi - exact).max())
    print("max |h Phi error| on [-8, 8]: %.2e" % np.abs(h * phi - h * exact).max())
