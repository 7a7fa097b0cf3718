#!/usr/bin/env python3
"""Generator of the Gaussian-tail coefficients in us_device.h (gauss_terms).

The kernels evaluate Q(x) = P(N(0,1) > x), x >= 0, as exp(-x^2/2) * R(x) with

    R(x) = Q(x) exp(x^2/2) = erfcx(x / sqrt 2) / 2   ~   t (c0 + c1 t + ... + c5 t^5),   t = 1 / (1 + p x),

so that Phi keeps RELATIVE accuracy far into the negative tail (GELU's x * Phi(x) needs it).  This script finds p and
the c_k by reweighted least squares (the weights grow where the relative error is largest, which drives the fit towards
the minimax one) on Chebyshev nodes of t over x in [0, 14], prints them, and compares them with the constants compiled
into the library.

    python fit_gauss_tail.py            # fit from scratch (about a minute), print, compare
    python fit_gauss_tail.py --check    # only evaluate the compiled-in constants against erfcx
"""
from __future__ import annotations

import os
import re
import sys

import numpy as np
from scipy import optimize, special

DEGREE = 6
X_MAX = 14.0


def nodes(p: float, count: int = 4000):
    t = 0.5 - 0.5 * np.cos(np.pi * (np.arange(count) + 0.5) / count)        # Chebyshev nodes in (0, 1)
    t = t[t > 1.0 / (1.0 + p * X_MAX)]
    x = (1.0 / t - 1.0) / p
    return t, x, 0.5 * special.erfcx(x / np.sqrt(2.0))


def fit(p: float, iters: int):
    """Coefficients for a given p and the largest relative error they leave."""
    t, _, R = nodes(p)
    A = np.stack([t ** (k + 1) for k in range(DEGREE)], 1)
    w = np.ones_like(t)
    for _ in range(iters):
        c, *_ = np.linalg.lstsq(A * (w / R)[:, None], w, rcond=None)
        rel = (A @ c) / R - 1.0
        w = w * (1.0 + 3.0 * np.abs(rel) / np.abs(rel).max())
        w /= w.mean()
    return c, float(np.abs(rel).max())


def compiled_constants():
    src = open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "us_device.h")).read()
    body = src[src.index("GaussTerms gauss_terms(float z)"):]
    p = float(re.search(r"constexpr float p = ([-0-9.e]+)f", body).group(1))
    cs = [float(re.search(rf"\bc{k} = ([-0-9.e]+)f", body).group(1)) for k in range(DEGREE)]
    return p, cs


def max_relative_error(p: float, cs, dtype=np.float64) -> float:
    """Largest relative error of t * poly(t) against erfcx(x / sqrt 2) / 2 on a dense grid of [0, 14], evaluated in `dtype`
    with the kernel's Horner order."""
    x = np.linspace(0.0, X_MAX, 200001)
    t = (1.0 / (1.0 + dtype(p) * x.astype(dtype))).astype(dtype)
    poly = np.full_like(t, dtype(cs[-1]))
    for c in cs[-2::-1]:
        poly = (poly * t + dtype(c)).astype(dtype)
    approx = (poly * t).astype(np.float64)
    return float(np.max(np.abs(approx / (0.5 * special.erfcx(x / np.sqrt(2.0))) - 1.0)))


def main():
    p0, c0 = compiled_constants()
    print("compiled in: p =", p0, "c =", c0)
    print("  max relative error on [0, 14]: %.2e (float64 evaluation), %.2e (float32 evaluation)"
          % (max_relative_error(p0, c0), max_relative_error(p0, c0, np.float32)))
    if "--check" in sys.argv:
        return
    res = optimize.minimize_scalar(lambda p: fit(p, 30)[1], bounds=(0.15, 0.6), method="bounded", options=dict(xatol=1e-5))
    c, err = fit(res.x, 200)
    print("fitted:      p = %.9f" % res.x, "c =", [float("%.8g" % v) for v in c], "max relative error %.2e" % err)
    print("  difference to the compiled-in constants: p %.1e, c %.1e" % (abs(res.x - p0), float(np.max(np.abs(c - np.array(c0))))))


if __name__ == "__main__":
    main()
