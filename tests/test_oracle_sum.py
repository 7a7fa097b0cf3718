"""Pins for the oracle's scaled sum (Table A.2 "Linear": alpha = n^-1/2, beta = 1), CPU only: numpy's float64 sum,
exact rationals, float64 autograd, unit variance of the output for unit-variance inputs."""
from fractions import Fraction

import numpy as np
import torch

import oracle
import synth


def _bits(a):
    return np.ascontiguousarray(a).view(np.uint16)


def test_factors_and_forward_against_numpy():
    assert oracle.sum_scales(1024) == (np.float32(1 / 32), np.float32(1.0))
    x = synth.normal(111, 1, (40, 200))
    y = oracle.sum_fwd(x)
    ref = (float(np.float32(200 ** -0.5)) * x.astype(np.float64).sum(axis=1)).astype(np.float16)
    assert np.max(np.abs(_bits(y).astype(np.int64) - _bits(ref).astype(np.int64))) <= 1      # numpy adds pairwise
    row = x[3]
    exact = Fraction(float(np.float32(200 ** -0.5))) * sum(Fraction(float(v)) for v in row)
    assert _bits(y)[3] == _bits(np.array([exact.numerator / exact.denominator], np.float64).astype(np.float16))[0]
    assert y.shape == (40,)


def test_small_integers_are_exact_and_the_sum_runs_over_the_last_axis():
    x = (np.arange(6)[:, None] * 10 + np.arange(16)[None, :]).astype(np.float16)          # x[i,j] = 10 i + j
    y = oracle.sum_fwd(x, alpha=0.25)
    assert np.array_equal(y.astype(np.float64), 0.25 * (160.0 * np.arange(6) + 120.0))


def test_backward_is_the_broadcast_gradient():
    g = synth.normal(112, 2, (12,))
    dx = oracle.sum_bwd(g, 48)
    assert dx.shape == (12, 48) and all(np.array_equal(_bits(dx[:, j]), _bits(g)) for j in range(48))
    xt = torch.zeros((12, 48), dtype=torch.float64, requires_grad=True)
    (xt.sum(dim=1) * torch.tensor(g.astype(np.float64))).sum().backward()
    assert np.array_equal(oracle.sum_bwd(g, 48, beta=0.5).astype(np.float64), (0.5 * xt.grad.numpy()).astype(np.float16).astype(np.float64))


def test_unit_variance():
    x = synth.normal(113, 1, (4096, 512))
    y = oracle.sum_fwd(x).astype(np.float64)
    assert abs(y.std() - 1.0) < 0.05 and abs(y.mean()) < 0.06
