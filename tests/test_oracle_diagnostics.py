"""Exponent histogram and cast SNR of the oracle (CPU only; Fig. 1, App. C, App. K, Sec. 3.1)."""
import math

import numpy as np
import pytest
from scipy import stats
from scipy.special import erf

import oracle
import synth
from oracle import E4M3, E5M2


def test_histogram_bins_on_hand_picked_values():
    v = np.array([0.0, -0.0, 6e-8, 2.0 ** -15, 2.0 ** -14, 1.0, 1.5, -1.999, 2.0, 65504.0, np.inf, -np.inf, np.nan], np.float16)
    h = oracle.exponent_histogram(v)
    want = np.zeros(oracle.HIST_BINS, np.uint64)
    want[0] = 2                      # both zeros
    want[2] = 2                      # FP16 subnormals: 2^-24 and 2^-15
    want[3] = 1                      # 2^-14, the smallest normal exponent
    want[3 + 14] = 3                 # 1.0, 1.5, -1.999: exponent 0
    want[3 + 15] = 1                 # 2.0
    want[3 + 29] = 1                 # 65504: exponent 15
    want[33] = 2
    want[34] = 1
    assert np.array_equal(h, want)
    v32 = np.array([1e-9, 70000.0, 3.0], np.float32)          # below the FP16 grid, above it, exponent 1
    h = oracle.exponent_histogram(v32)
    assert h[1] == 1 and h[33] == 1 and h[3 + 15] == 1 and h.sum() == 3


def test_histogram_of_a_unit_normal_tensor_matches_the_gaussian_bin_probabilities():
    """P(2^e <= |x| < 2^(e+1)) = erf(2^(e+1)/sqrt 2) - erf(2^e/sqrt 2); App. C: the central 90 % of |N(0,1)| lies in
    [2^-4, 2^1] (exponents -4 .. 0)."""
    n = 1 << 22
    x = synth.normal(127, 1, (n,))
    h = oracle.exponent_histogram(x).astype(np.float64)
    assert h.sum() == n
    for e in range(-8, 2):
        p = erf(2.0 ** (e + 1) / math.sqrt(2)) - erf(2.0 ** e / math.sqrt(2))
        assert abs(h[3 + e + 14] / n - p) < 4 * math.sqrt(p / n) + 1e-6, e
    central = h[3 + 10: 3 + 15].sum() / n
    assert 0.90 < central < 0.925                      # exact: erf(2/sqrt2) - erf(2^-4/sqrt2) = 0.9047
    # numpy's own exponent extraction on the same data
    m, ex = np.frexp(np.abs(x[x != 0]).astype(np.float64))
    ex = ex - 1
    for e in range(-14, 3):
        assert h[3 + e + 14] == np.sum(ex == e)


def _snr_closed_form(fmt_bits_m, emin, fmax, sigma):
    """E[(q(X)-X)^2] for X ~ N(0, sigma^2) and round-to-nearest onto the grid {k 2^(e-M)} with saturation at fmax,
    by integrating (x - c)^2 phi(x) over every rounding interval in closed form."""
    M = fmt_bits_m
    pts = [0.0]
    e = emin
    step = 2.0 ** (emin - M)
    v = step
    while v <= fmax + 1e-30:
        pts.append(v)
        ex = max(math.floor(math.log2(v * (1 + 1e-15))), emin)
        v += 2.0 ** (ex - M)
    pts = np.array(pts)
    mids = (pts[1:] + pts[:-1]) / 2
    lo = np.concatenate([[0.0], mids])
    hi = np.concatenate([mids, [np.inf]])
    s = sigma
    def seg(c, a, b):   # int_a^b (x-c)^2 N(x; 0, s^2) dx, closed form
        F = lambda t: stats.norm.cdf(t / s) if np.isfinite(t) else 1.0
        f = lambda t: stats.norm.pdf(t / s) * s if np.isfinite(t) else 0.0      # s^2 * pdf_s(t)
        tf = lambda t: t * f(t) if np.isfinite(t) else 0.0
        i0 = F(b) - F(a)
        i1 = -(f(b) - f(a))                                                     # int x N dx
        i2 = s * s * i0 - (tf(b) - tf(a))                                       # int x^2 N dx
        return i2 - 2 * c * i1 + c * c * i0
    err = 2 * sum(seg(c, a, b) for c, a, b in zip(pts, lo, hi))
    return sigma * sigma / err


@pytest.mark.parametrize("fmt,M,emin,fmax", [(E4M3, 3, -6, 448.0), (E5M2, 2, -14, 57344.0)])
@pytest.mark.parametrize("sigma", [1.0, 2.0 ** -7, 64.0])
def test_snr_against_the_closed_form_integral(fmt, M, emin, fmax, sigma):
    """Sampled SNR of 4 Mi normal values against the exact expectation (rounding, subnormal and clipping
    regimes: sigma = 1, 2^-7, 64)."""
    n = 1 << 22
    x = synth.normal(131, 1, (n,), sigma=sigma).astype(np.float32)
    s0, s1 = oracle.cast_snr(x, fmt)
    want = _snr_closed_form(M, emin, fmax, sigma)
    assert abs((s0 / s1) / want - 1) < 0.02, (s0 / s1, want)


def test_snr_scale_and_special_values():
    x = synth.normal(137, 1, (1 << 16,)).astype(np.float32)
    a = oracle.cast_snr(x, E4M3, 1.0)
    b = oracle.cast_snr((x * 8).astype(np.float32), E4M3, 0.125)             # power-of-two rescaling is exact
    assert abs(a[0] * 64 - b[0]) < 1e-6 * b[0] and abs(a[1] * 64 - b[1]) < 1e-6 * b[1]
    # representable values carry no error; NaN is skipped; saturation counts as error
    exact = np.array([1.0, -0.5, 448.0, 0.0], np.float32)
    assert oracle.cast_snr(exact, E4M3) == (1.0 + 0.25 + 448.0 ** 2, 0.0)
    assert oracle.cast_snr(np.array([np.nan, 2.0], np.float32), E4M3) == (4.0, 0.0)
    assert oracle.cast_snr(np.array([1000.0], np.float32), E4M3) == (1e6, (1000.0 - 448.0) ** 2)
