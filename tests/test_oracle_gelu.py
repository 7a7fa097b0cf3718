"""Pins for the oracle's unit-scaled GELU (CPU only): scipy's normal CDF as an independent Phi, the
constants printed in Table A.2, quadrature of the scale-selection rule, finite differences."""
import math
import os

import numpy as np
from scipy import integrate, special

import oracle
import synth
from oracle import F16, F32


def _printed():
    rows = {}
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "table_a2_factors.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, a, b = line.split()
        rows[name] = (float(a), float(b))
    return rows


def _rule(f, df):
    """alpha = 1/std f(z), beta = 1/rms f'(z), z ~ N(0,1) (Sec. 5.2 'Selecting scaling factors')."""
    pdf = lambda z: math.exp(-0.5 * z * z) / math.sqrt(2 * math.pi)
    E = lambda g: integrate.quad(lambda z: g(z) * pdf(z), -12, 12, epsabs=1e-13, epsrel=1e-13)[0]
    mean, second, dsecond = E(f), E(lambda z: f(z) ** 2), E(lambda z: df(z) ** 2)
    return 1 / math.sqrt(second - mean ** 2), 1 / math.sqrt(dsecond)


def test_scale_rule_reproduces_table_a2():
    printed = _printed()
    Phi = lambda z: float(special.ndtr(z))
    pdf = lambda z: math.exp(-0.5 * z * z) / math.sqrt(2 * math.pi)
    a, b = _rule(lambda z: z * Phi(z), lambda z: Phi(z) + z * pdf(z))
    assert round(a, 3) == printed["gelu"][0] and round(b, 3) == printed["gelu"][1]
    ag, bg = oracle.gelu_scales()
    assert abs(float(ag) - a) < 1e-6 and abs(float(bg) - b) < 1e-6      # closed forms == quadrature
    # the same rule gives the analytic ReLU row and the other printed rows: pins the reading of the rule
    a, b = _rule(lambda z: max(z, 0.0), lambda z: 1.0 if z > 0 else 0.0)
    assert abs(a - math.sqrt(2 / (1 - 1 / math.pi))) < 1e-6 and abs(b - math.sqrt(2)) < 1e-6
    a, b = _rule(math.tanh, lambda z: 1 - math.tanh(z) ** 2)
    assert abs(a - printed["tanh"][0]) < 1e-3 and abs(b - printed["tanh"][1]) < 1e-3
    sg = lambda z: 1 / (1 + math.exp(-z))
    a, b = _rule(sg, lambda z: sg(z) * (1 - sg(z)))
    assert abs(a - printed["sigmoid"][0]) < 2e-3 and abs(b - printed["sigmoid"][1]) < 2e-3


def test_gelu_fwd_all_fp16_inputs_vs_scipy():
    h = np.arange(65536, dtype=np.uint32).astype(np.uint16).view(np.float16)
    h = h[np.isfinite(h.astype(np.float32))]
    ag = oracle.gelu_scales()[0]
    z = h.astype(np.float64)
    with np.errstate(over="ignore"):
        want = (np.float64(ag) * z * special.ndtr(z)).astype(np.float16)
    got = oracle.gelu_fwd(h, ag)
    # two independent Phi implementations may differ in the last double bit: allow FP16 ties only
    diff = got.view(np.uint16).astype(np.int32) - want.view(np.uint16).astype(np.int32)
    assert np.count_nonzero(diff) <= 2 and np.max(np.abs(diff)) <= 1
    assert oracle.gelu_fwd(np.zeros(1, np.float16), ag)[0] == 0
    big = np.array([8.0, 20.0, 100.0], np.float16)
    assert np.array_equal(oracle.gelu_fwd(big, 1.0), big)                     # gelu(z) -> z
    neg = oracle.gelu_fwd(np.array([-6.0, -12.0, -40.0], np.float16), 1.0).astype(np.float64)
    assert np.all(neg <= 0) and np.all(np.abs(neg) < 1e-7)                     # gelu(z) -> -0
    # negative tail keeps relative accuracy (erfc form): z = -5
    v = float(oracle.gelu_fwd(np.array([-5.0], np.float32), 1.0)[0])
    assert abs(v / (-5.0 * 2.8665157187919333e-07) - 1) < 1e-6                # Phi(-5) to 17 digits


def test_gelu_bwd_vs_finite_difference_and_scipy():
    z = synth.normal(53, 1, (1 << 14,), sigma=1.5, dtype=np.float32)
    g = synth.normal(53, 2, (1 << 14,), dtype=np.float32)
    bg = oracle.gelu_scales()[1]
    got = oracle.gelu_bwd(z, g, bg).astype(np.float64)
    zd = z.astype(np.float64)
    f = lambda t: t * special.ndtr(t)
    eps = 1e-5
    fd = (f(zd + eps) - f(zd - eps)) / (2 * eps)
    want = np.float64(bg) * fd * g.astype(np.float64)
    assert np.max(np.abs(got - want)) < 1e-6
    assert abs(float(oracle.gelu_bwd(np.zeros(1, np.float32), np.ones(1, np.float32), 1.0)[0]) - 0.5) < 1e-7
    # FP16 storage: one rounding of the double result
    z16, g16 = z.astype(np.float16), g.astype(np.float16)
    got16 = oracle.gelu_bwd(z16, g16, bg)
    zd, gd = z16.astype(np.float64), g16.astype(np.float64)
    pdf = np.exp(-0.5 * zd * zd) / math.sqrt(2 * math.pi)
    want16 = (np.float64(bg) * (special.ndtr(zd) + zd * pdf) * gd).astype(np.float16)
    diff = got16.view(np.uint16).astype(np.int32) - want16.view(np.uint16).astype(np.int32)
    assert np.count_nonzero(diff) <= 2 and np.max(np.abs(diff)) <= 1


def test_unit_scaled_gelu_has_unit_std_and_unit_rms_gradient():
    z = synth.normal(59, 1, (1 << 20,))
    g = synth.normal(59, 2, (1 << 20,))
    ag, bg = oracle.gelu_scales()
    h = oracle.gelu_fwd(z, ag).astype(np.float64)
    gz = oracle.gelu_bwd(z, g, bg).astype(np.float64)
    assert abs(h.std() - 1.0) < 0.01
    assert abs(h.mean() - float(ag) / (2 * math.sqrt(math.pi))) < 0.005        # mean is not zero (App. E.1 remark)
    assert abs(np.sqrt(np.mean(gz ** 2)) - 1.0) < 0.01
