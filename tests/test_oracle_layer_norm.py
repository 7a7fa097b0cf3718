"""Scaled layer norm of the oracle (CPU only; Table A.2 "Other")."""
import math

import numpy as np
import pytest
import torch

import oracle
import synth


def _inputs(b, n, seed, sigma=1.0, shift=0.0):
    X = (synth.normal(seed, 1, (b, n), sigma=sigma).astype(np.float32) + shift).astype(np.float16)
    w = (1.0 + 0.25 * synth.normal(seed, 2, (n,)).astype(np.float32)).astype(np.float16)
    c = (0.1 * synth.normal(seed, 3, (n,)).astype(np.float32)).astype(np.float16)
    G = synth.normal(seed, 4, (b, n))
    return X, w, c, G


def test_scale_rule():
    assert oracle.layer_norm_scales(4096) == (1.0, 1.0, np.float32(1 / 64))


def test_forward_against_the_library_routine():
    """torch.nn.functional.layer_norm in float64 (biased variance, the same definition; eps inside the root)."""
    X, w, c, _ = _inputs(64, 96, 103, sigma=2.0, shift=0.5)
    for eps in (0.0, 1e-5):
        Y, mean, rstd = oracle.layer_norm_fwd(X, w, c, eps)
        t = lambda a: torch.from_numpy(a.astype(np.float64))
        ref = torch.nn.functional.layer_norm(t(X), (96,), t(w), t(c), eps).numpy()
        assert np.array_equal(Y.view(np.uint16), ref.astype(np.float16).view(np.uint16))
        assert np.allclose(mean, X.astype(np.float64).mean(1), rtol=0, atol=1e-13)
        assert np.allclose(rstd, 1 / np.sqrt(X.astype(np.float64).var(1) + eps), rtol=1e-12)


def test_normalised_rows_and_identity_parameters():
    X, _, _, _ = _inputs(128, 256, 107, sigma=5.0, shift=-3.0)
    one, zero = np.ones(256, np.float16), np.zeros(256, np.float16)
    Y, _, _ = oracle.layer_norm_fwd(X, one, zero)
    y = Y.astype(np.float64)
    assert np.max(np.abs(y.mean(1))) < 2e-3 and np.max(np.abs(y.std(1) - 1.0)) < 2e-3
    # scaling a row leaves the output unchanged (powers of two are exact in FP16)
    Y2, _, _ = oracle.layer_norm_fwd((X.astype(np.float32) * 0.25).astype(np.float16), one, zero)
    assert np.array_equal(Y, Y2)


def test_backward_against_autograd_of_the_library_routine():
    """float64 autograd through torch's layer_norm; the scaled backward multiplies dw, dc by b^-1/2 and dX by 1."""
    b, n = 48, 80
    X, w, c, G = _inputs(b, n, 109, sigma=1.5, shift=0.3)
    for eps in (0.0, 1e-5):
        tx = torch.from_numpy(X.astype(np.float64)).requires_grad_()
        tw = torch.from_numpy(w.astype(np.float64)).requires_grad_()
        tc = torch.from_numpy(c.astype(np.float64)).requires_grad_()
        y = torch.nn.functional.layer_norm(tx, (n,), tw, tc, eps)
        y.backward(torch.from_numpy(G.astype(np.float64)))
        dX, dw, dc = oracle.layer_norm_bwd(X, w, G, eps)
        beta = float(oracle.layer_norm_scales(b)[2])
        assert np.array_equal(dX.view(np.uint16), tx.grad.numpy().astype(np.float16).view(np.uint16))
        assert np.array_equal(dw.view(np.uint16), (beta * tw.grad.numpy()).astype(np.float16).view(np.uint16))
        assert np.array_equal(dc.view(np.uint16), (beta * tc.grad.numpy()).astype(np.float16).view(np.uint16))


def test_gradient_identities_and_unit_variance():
    """dX of every row sums to zero and is orthogonal to the normalised row (the two projections of f_grad);
    with unit-variance inputs, unit weights and an independent unit gradient: Var(Y) = 1, Var(dX) = 1 - 2/n,
    Var(dw) = Var(dc) = 1 after the b^-1/2 factor."""
    b, n = 2048, 512
    X, _, _, G = _inputs(b, n, 113)
    one, zero = np.ones(n, np.float16), np.zeros(n, np.float16)
    Y, mean, rstd = oracle.layer_norm_fwd(X, one, zero)
    dX, dw, dc = oracle.layer_norm_bwd(X, one, G)
    xh = (X.astype(np.float64) - mean[:, None]) * rstd[:, None]
    d = dX.astype(np.float64)
    assert np.max(np.abs(d.sum(1))) < 0.15 and np.max(np.abs((d * xh).sum(1))) < 0.15       # FP16 rounding of 512 terms
    v = lambda a: float(np.var(a.astype(np.float64)))
    assert abs(v(Y) - 1.0) < 0.01 and abs(v(dX) - (1 - 2 / n)) < 0.02
    assert abs(v(dw) - 1.0) < 0.15 and abs(v(dc) - 1.0) < 0.15                               # 512 samples each


def test_zero_variance_row_follows_the_printed_formula():
    """No epsilon in the paper's formula: a constant row divides by zero (inf/NaN), an epsilon makes it the bias."""
    X = np.full((1, 32), 3.0, np.float16)
    w, c = np.ones(32, np.float16), np.full(32, 0.5, np.float16)
    Y, _, rstd = oracle.layer_norm_fwd(X, w, c, 0.0)
    assert np.isinf(rstd[0]) and np.isnan(Y.astype(np.float32)).all()
    Y, _, _ = oracle.layer_norm_fwd(X, w, c, 1e-5)
    assert np.all(Y == np.float16(0.5))
