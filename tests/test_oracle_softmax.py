"""Pins for the oracle's scaled softmax and softmax cross-entropy (CPU only): scipy's float64 softmax / logsumexp,
closed forms (two classes = logistic function; a constant row), the worked variance of App. G "Softmax
cross-entropy", torch's float64 autograd, invariances, and the scale the paper's rule gives the outputs."""
import numpy as np
import pytest
import torch
from scipy.special import logsumexp, softmax

import oracle
import synth


def _f16(a):
    return np.asarray(a, np.float64).astype(np.float16)


def _bits(a):
    return np.ascontiguousarray(a).view(np.uint16)


def test_scale_factors_table_a2():
    assert oracle.softmax_scales(128) == (np.float32(128), np.float32(128))
    assert oracle.softmax_xent_scale(30522) == np.float32(30522 / np.sqrt(30521.0))
    assert abs(float(oracle.softmax_xent_scale(2)) - 2.0) < 1e-7


def test_forward_against_scipy_and_row_sums():
    x = synth.normal(81, 1, (64, 200), sigma=2.0)
    y = oracle.softmax_fwd(x)                                       # alpha = s = 200
    ref = _f16(200.0 * softmax(x.astype(np.float64), axis=1))
    assert np.array_equal(_bits(y), _bits(ref))
    assert np.allclose(y.astype(np.float64).sum(axis=1), 200.0, rtol=1e-3)
    # an explicit alpha and an input factor (temperature 1/s1)
    y2 = oracle.softmax_fwd(x, alpha=1.0, s1=0.5)
    assert np.array_equal(_bits(y2), _bits(_f16(softmax(0.5 * x.astype(np.float64), axis=1))))


def test_closed_forms():
    # a constant row: exactly alpha / s in every place, whatever the constant
    for c in (0.0, -3.5, 11.0):
        x = np.full((2, 64), c, np.float16)
        assert np.all(oracle.softmax_fwd(x) == np.float16(1.0))
    # two classes: softmax([a, b])_0 = 1 / (1 + exp(b - a))
    a, b = 0.75, -1.25
    y = oracle.softmax_fwd(np.array([[a, b]], np.float16), alpha=1.0)
    assert np.array_equal(_bits(y), _bits(_f16([[1 / (1 + np.exp(b - a)), 1 / (1 + np.exp(a - b))]])))
    # shift invariance, and no overflow for large inputs (the maximum is subtracted)
    x = synth.normal(82, 1, (8, 48))
    big = (x.astype(np.float64) + 1000.0).astype(np.float16)          # exactly representable shifts of the rounded values
    assert np.array_equal(_bits(oracle.softmax_fwd(big)), _bits(_f16(48.0 * softmax(big.astype(np.float64), axis=1))))
    assert np.all(np.isfinite(oracle.softmax_fwd(np.array([[60000.0, 60000.0, -60000.0, 0.0]], np.float16))))
    # NaN anywhere in a row makes the row NaN
    xn = np.array([[0.0, np.nan, 1.0, 2.0]], np.float16)
    assert np.all(np.isnan(oracle.softmax_fwd(xn)))


def test_backward_against_autograd_and_identities():
    rows, s = 32, 96
    x = synth.normal(83, 1, (rows, s), sigma=1.5)
    g = synth.normal(83, 2, (rows, s))
    dx = oracle.softmax_bwd(x, g, beta=3.0, s1=0.5)
    xt = torch.tensor(x.astype(np.float64), requires_grad=True)
    (torch.softmax(0.5 * xt, dim=1) * torch.tensor(g.astype(np.float64))).sum().backward()
    assert np.array_equal(_bits(dx), _bits(_f16(3.0 * xt.grad.numpy())))
    # the gradient of a softmax sums to zero over the row; a constant added to g changes nothing
    assert np.all(np.abs(dx.astype(np.float64).sum(axis=1)) < 0.05)
    g2 = (g.astype(np.float64) + 2.0).astype(np.float16)
    d2 = oracle.softmax_bwd(x, g2, beta=3.0, s1=0.5)
    assert np.max(np.abs(d2.astype(np.float64) - dx.astype(np.float64))) < 0.02
    # constant row: p = 1/s, so dx = (beta / s) (g - mean g): with beta = s a unit-variance g gives unit variance back
    # (s a power of two, so that beta / s = 1 and p = 1/s carry no rounding of their own)
    gc = synth.normal(83, 3, (rows, 128))
    dc = oracle.softmax_bwd(np.zeros((rows, 128), np.float16), gc)
    ref = gc.astype(np.float64) - gc.astype(np.float64).mean(axis=1, keepdims=True)
    assert np.max(np.abs(_bits(dc).astype(np.int64) - _bits(_f16(ref)).astype(np.int64))) <= 1
    assert np.mean(_bits(dc) != _bits(_f16(ref))) < 2e-3            # a different order of the additions in the mean


def test_scale_of_the_outputs_for_unit_normal_inputs():
    s = 512
    x = synth.normal(84, 1, (256, s))
    g = synth.normal(84, 2, (256, s))
    y = oracle.softmax_fwd(x).astype(np.float64)
    assert abs(y.mean() - 1.0) < 1e-3                                # about a vector of ones (App. G): the mean is one exactly
    # s p_j ~ exp(x_j - 1/2) for large s: second moment E exp(2x - 1) = e
    assert abs(np.mean(y ** 2) - np.e) < 0.25
    d = oracle.softmax_bwd(x, g).astype(np.float64)
    assert abs(d.mean()) < 0.02 and abs(d.std() - np.sqrt(np.e)) < 0.15   # the same factor reaches the gradient
    # for inputs of small variance both are at unit scale, the case the paper's rule is derived for
    xs = synth.normal(84, 3, (256, s), sigma=0.125)
    assert abs(oracle.softmax_fwd(xs).astype(np.float64).std() - 0.125) < 0.02
    assert abs(oracle.softmax_bwd(xs, g).astype(np.float64).std() - 1.0) < 0.03


def test_xent_against_scipy_and_autograd():
    rows, s = 48, 120
    x = synth.normal(85, 1, (rows, s), sigma=2.0)
    t = (np.arange(rows) * 7) % s
    loss, dx = oracle.softmax_xent(x, t, beta=2.0, s1=0.5)
    xd = 0.5 * x.astype(np.float64)
    assert np.allclose(loss, logsumexp(xd, axis=1) - xd[np.arange(rows), t], rtol=1e-13, atol=1e-13)
    xt = torch.tensor(x.astype(np.float64), requires_grad=True)
    torch.nn.functional.cross_entropy(0.5 * xt, torch.tensor(t), reduction="sum").backward()
    assert np.array_equal(_bits(dx), _bits(_f16(2.0 * xt.grad.numpy())))
    # rows without a label
    t2 = t.copy(); t2[3] = -1; t2[5] = s
    loss2, dx2 = oracle.softmax_xent(x, t2, beta=2.0, s1=0.5)
    assert loss2[3] == 0 and loss2[5] == 0 and not dx2[3].any() and not dx2[5].any()
    keep = np.ones(rows, bool); keep[[3, 5]] = False
    assert np.array_equal(loss2[keep], loss[keep]) and np.array_equal(_bits(dx2[keep]), _bits(dx[keep]))


@pytest.mark.parametrize("s", [2, 16, 1024, 30528])
def test_xent_worked_example_of_app_g(s):
    """Uniform softmax output: the gradient is (1 - s)/s at the target and 1/s elsewhere, mean 0, variance (s - 1)/s^2,
    so beta = s / sqrt(s - 1) brings it to variance 1."""
    x = np.zeros((1, s), np.float16)
    _, raw = oracle.softmax_xent(x, [s // 3], beta=1.0)
    raw = raw.astype(np.float64)[0]
    assert abs(raw[s // 3] - (1 - s) / s) <= 2.0 ** -11 and np.allclose(np.delete(raw, s // 3), 1 / s, rtol=2.0 ** -10)
    _, dx = oracle.softmax_xent(x, [s // 3])
    d = dx.astype(np.float64)[0]
    assert abs(d.mean()) < 1e-3 and abs(np.mean(d ** 2) - 1.0) < 2e-3
    loss, _ = oracle.softmax_xent(x, [0])
    assert abs(loss[0] - np.log(s)) < 1e-12
