"""relu / tanh / sigmoid of the oracle (CPU only; Table A.2 "Activations", App. E.1, App. H)."""
import math

import numpy as np
import pytest
from scipy import integrate, stats

import oracle
import synth
from oracle import GELU, RELU, SIGMOID, TANH


def _golden():
    rows = {}
    for line in open(__file__.rsplit("/", 1)[0] + "/golden/table_a2_factors.txt"):
        p = line.split("#")[0].split()
        if len(p) == 3:
            rows[p[0]] = (float(p[1]), float(p[2]))
    return rows


def test_scale_factors_match_the_printed_table():
    """Table A.2 prints relu analytically and gelu / tanh / sigmoid to four significant digits, found "empirically"
    (by sampling): the exact integrals agree to half a unit of the last digit, except sigmoid's alpha
    (4.8013 against the printed 4.802: 1.4e-4 relative, the size of a sampling error)."""
    g = _golden()
    for name, kind in (("gelu", GELU), ("tanh", TANH), ("sigmoid", SIGMOID)):
        a, b = oracle.act_scales(kind)
        assert abs(float(a) / g[name][0] - 1) < 3.5e-4 and abs(float(b) / g[name][1] - 1) < 3.5e-4, name
    a, b = oracle.act_scales(RELU)
    assert abs(float(a) - math.sqrt(2 / (1 - 1 / math.pi))) < 1e-6 and abs(float(b) - math.sqrt(2)) < 1e-6


@pytest.mark.parametrize("kind,f,df", [
    (TANH, np.tanh, lambda x: 1 - np.tanh(x) ** 2),
    (SIGMOID, lambda x: 1 / (1 + np.exp(-x)), lambda x: np.exp(-x) / (1 + np.exp(-x)) ** 2),
])
def test_quadrature_of_the_scale_rule_by_an_independent_integrator(kind, f, df):
    """scipy's adaptive quadrature instead of Gauss-Hermite nodes."""
    pdf = stats.norm.pdf
    m = integrate.quad(lambda x: f(x) * pdf(x), -12, 12)[0]
    v = integrate.quad(lambda x: f(x) ** 2 * pdf(x), -12, 12)[0] - m * m
    d2 = integrate.quad(lambda x: df(x) ** 2 * pdf(x), -12, 12)[0]
    a, b = oracle.act_scales(kind)
    assert abs(float(a) - v ** -0.5) < 1e-6 and abs(float(b) - d2 ** -0.5) < 1e-6


@pytest.mark.parametrize("kind", [GELU, RELU, TANH, SIGMOID])
def test_unit_variance_after_scaling(kind):
    z = synth.normal(89, 1, (1024, 1024))
    g = synth.normal(89, 2, (1024, 1024))
    a, b = oracle.act_scales(kind)
    assert abs(np.std(oracle.act_fwd(z, kind, a).astype(np.float64)) - 1.0) < 0.01
    gz = oracle.act_bwd(z, g, kind, b).astype(np.float64)
    assert abs(np.sqrt(np.mean(gz ** 2)) - 1.0) < 0.01


def test_values_against_numpy_and_special_points():
    z = np.concatenate([synth.normal(97, 1, (4096,), sigma=3.0), np.array([0.0, -0.0, 1.0, -1.0, 11.0, -11.0, 6e-8, 65504, -65504], np.float16)])
    g = np.concatenate([synth.normal(97, 2, (4096,)), np.ones(9, np.float16)])
    z64, g64 = z.astype(np.float64), g.astype(np.float64)
    cases = {
        RELU: (np.maximum(z64, 0), (z64 > 0).astype(np.float64)),
        TANH: (np.tanh(z64), 1 / np.cosh(np.clip(z64, -300, 300)) ** 2),
        SIGMOID: (1 / (1 + np.exp(-z64)), np.exp(-np.abs(z64)) / (1 + np.exp(-np.abs(z64))) ** 2),
        GELU: (z64 * stats.norm.cdf(z64), stats.norm.cdf(z64) + z64 * stats.norm.pdf(z64)),
    }
    for kind, (f, df) in cases.items():
        s = np.float32(1.37)
        h = oracle.act_fwd(z, kind, s).astype(np.float64)
        with np.errstate(over="ignore"):
            want = (np.float64(s) * f).astype(np.float16).astype(np.float64)
        fin = np.isfinite(want)                                # 1.37 * 65504 overflows FP16 on both sides
        assert np.array_equal(h[~fin], want[~fin]), kind
        assert np.max(np.abs(h[fin] - want[fin]) / np.maximum(np.abs(want[fin]), 1e-4)) < 1e-3, kind   # at most a rounding flip
        assert np.mean(h[fin] != want[fin]) < 2e-3, kind
        gz = oracle.act_bwd(z, g, kind, s).astype(np.float64)
        want = (np.float64(s) * df * g64).astype(np.float16).astype(np.float64)
        assert np.mean(gz != want) < 2e-3, kind
    # gelu through the generic entry equals the dedicated one bit for bit
    a, b = oracle.gelu_scales()
    assert np.array_equal(oracle.act_fwd(z, GELU, a).view(np.uint16), oracle.gelu_fwd(z, a).view(np.uint16))
    fin = np.isfinite(z.astype(np.float32)) & (np.abs(z.astype(np.float32)) < 60000)
    assert np.array_equal(oracle.act_bwd(z, g, GELU, b)[fin], oracle.gelu_bwd(z, g, b)[fin])
    # special points
    one = np.ones(1, np.float16)
    assert oracle.act_bwd(np.zeros(1, np.float16), one, RELU, 1.0)[0] == 0.0          # relu'(0) = 0
    assert oracle.act_fwd(np.zeros(1, np.float16), SIGMOID, 1.0)[0] == 0.5
    assert oracle.act_bwd(np.zeros(1, np.float16), one, SIGMOID, 1.0)[0] == 0.25
    assert oracle.act_bwd(np.zeros(1, np.float16), one, TANH, 1.0)[0] == 1.0


def test_aligned_form_is_the_plain_function_of_the_scaled_input():
    """App. H: f_hat(x) = f(s1 x) s2.  With FP16 storage s1*z is not rounded before f is applied."""
    z = synth.normal(101, 1, (2048,))
    s1, s2 = 0.75, 2.5
    for kind, f in ((TANH, np.tanh), (RELU, lambda x: np.maximum(x, 0))):
        got = oracle.act_fwd(z, kind, s2, s1).astype(np.float64)
        want = (np.float64(np.float32(s2)) * f(np.float64(np.float32(s1)) * z.astype(np.float64))).astype(np.float16).astype(np.float64)
        assert np.mean(got != want) < 2e-3
