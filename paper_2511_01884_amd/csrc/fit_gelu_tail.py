"""Fits the degree-5 polynomial P with Phi(-x) ~ 2^P(x), x >= 0, used by gelu_erf in ff_device.hpp.

Phi is the standard normal distribution function.  The fit minimises the largest error of
x * 2^P(x) against x * Phi(-x) (the error it causes in GELU) by iteratively reweighted least squares
on a dense grid, then evaluates the result in float32 arithmetic over z in [-12, 12] and prints the
coefficients, the largest error, and the stationary points of P (none may be real and positive:
2^P must keep falling beyond the fitted range).  Needs numpy and scipy; not used at run time.
"""
import numpy as np
from scipy.special import erfc, log_ndtr

DEGREE, RANGE = 5, 5.5


def fit(deg=DEGREE, X=RANGE, iters=200, n=20001):
    x = np.linspace(0, X, n)
    f = log_ndtr(-x) / np.log(2.0)
    weight = x * np.exp(log_ndtr(-x)) * np.log(2.0) + 1e-12   # error of g per unit error of the exponent
    lawson = np.ones_like(x)
    V = np.vander(x / X, deg + 1, increasing=True)
    for _ in range(iters):
        w = np.sqrt(lawson) * weight
        c, *_ = np.linalg.lstsq(V * w[:, None], f * w, rcond=None)
        e = np.abs((V @ c - f) * weight)
        lawson = lawson * (e / e.max() + 1e-3)
        lawson /= lawson.sum()
    return c / X ** np.arange(deg + 1)


def max_error_float32(c):
    c32 = c.astype(np.float32)
    z = np.linspace(-12, 12, 2400001).astype(np.float32)
    x = np.abs(z)
    p = np.full_like(x, c32[-1])
    for k in range(len(c32) - 2, -1, -1):
        p = (p * x + c32[k]).astype(np.float32)
    g = np.maximum(z, 0).astype(np.float64) - x.astype(np.float64) * np.exp2(p.astype(np.float64))
    z64 = z.astype(np.float64)
    err = np.abs(g - 0.5 * z64 * erfc(-z64 / np.sqrt(2)))
    return float(err.max()), float(z[err.argmax()])


if __name__ == "__main__":
    c = fit()
    print("coefficients, constant term first:", ["%.9g" % v for v in c])
    print("largest error of g, at z:", max_error_float32(c))
    print("stationary points of P:", np.polynomial.polynomial.polyroots(np.polynomial.polynomial.polyder(c)))
