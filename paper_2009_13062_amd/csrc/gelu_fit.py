#!/usr/bin/env python3
"""Fit of the GELU constants in nf_common.h (gelu_erf).

GELU(v) = v Phi(v) is evaluated with one transcendental: for a = |v|, 1 - Phi(a) = 2^g(a) with
g(a) = log2(1 - Phi(a)), a smooth function that a degree-6 polynomial replaces on [0, 8]; Phi(v) = 1 - 2^g for
v >= 0 and 2^g for v < 0.  The fit minimises the maximum of the resulting GELU error |a (2^p(a) - 2^g(a))|
(iteratively re-weighted least squares).  Needs numpy and scipy only.

    python gelu_fit.py            prints the coefficients (constant term first) and the achieved error
"""
from math import log

import numpy as np
from scipy.special import log_ndtr, ndtr

A = 8.0
DEGREE = 6


def fit(degree=DEGREE, iters=60):
    a = np.linspace(0.0, A, 20001)
    g = log_ndtr(-a) / log(2.0)                    # log2(1 - Phi(a))
    w = np.maximum(a * 2.0 ** g, 1e-12)            # d(GELU error) / d(g error), up to ln 2
    W = w.copy()
    V = np.vander(a, degree + 1, increasing=True)
    c = None
    for _ in range(iters):
        c, *_ = np.linalg.lstsq(V * W[:, None], g * W, rcond=None)
        err = np.abs((V @ c - g) * w)
        W = W * (1 + 4 * err / err.max())
        W /= W.max()
    return [float(np.float32(x)) for x in c]


def gelu_poly_f32(v, c):
    """gelu_erf of nf_common.h in numpy float32 arithmetic (separate multiply and add instead of the fused
    multiply-add: the difference is below the last digit of the error reported here)."""
    v = np.asarray(v, np.float32)
    a = np.minimum(np.abs(v), np.float32(A))
    p = np.full_like(a, np.float32(c[-1]))
    for k in range(len(c) - 2, -1, -1):
        p = (p * a + np.float32(c[k])).astype(np.float32)
    tail = np.exp2(p).astype(np.float32)
    return (v * np.where(v < 0, tail, np.float32(1) - tail)).astype(np.float32)


def max_abs_error(c, lo=-12.0, hi=12.0, n=2000001):
    v = np.linspace(lo, hi, n)
    return float(np.abs(gelu_poly_f32(v, c).astype(np.float64) - v * ndtr(v)).max())


if __name__ == "__main__":
    coef = fit()
    print("coefficients (a^0 .. a^%d):" % DEGREE)
    for x in coef:
        print("  %r" % x)
    print("max |gelu_poly - gelu| on [-12, 12] in float32 arithmetic: %.3e" % max_abs_error(coef))
