"""GPU parity: scaled layer norm forward / backward against the oracle (Table A.2 "Other")."""
import numpy as np
import pytest
import torch

import oracle
import paper_2303_11257_amd as us
import synth
from gpu_util import DEV, assert_close, empty, ptr, stream, to_dev, to_np

pytestmark = pytest.mark.gpu
O = oracle


def _inputs(b, n, seed, sigma=1.0, shift=0.0):
    X = (synth.normal(seed, 1, (b, n), sigma=sigma).astype(np.float32) + shift).astype(np.float16)
    w = (1.0 + 0.25 * synth.normal(seed, 2, (n,)).astype(np.float32)).astype(np.float16)
    c = (0.1 * synth.normal(seed, 3, (n,)).astype(np.float32)).astype(np.float16)
    G = synth.normal(seed, 4, (b, n))
    return X, w, c, G


def _run(X, w, c, G, eps, beta=0.0):
    b, n = X.shape
    tX, tw, tc, tG = to_dev(X), to_dev(w), to_dev(c), to_dev(G)
    Y, dX, dw, dc = empty((b, n), np.float16), empty((b, n), np.float16), empty((n,), np.float16), empty((n,), np.float16)
    us.layer_norm_fwd(ptr(tX), ptr(tw), ptr(tc), ptr(Y), b, n, eps, stream())
    wsb = us.layer_norm_workspace_bytes(b, n)
    ws = torch.full((wsb,), 0x5A, dtype=torch.uint8, device=DEV)
    us.layer_norm_bwd(ptr(tX), ptr(tw), ptr(tG), ptr(dX), ptr(dw), ptr(dc), b, n, eps, beta, ptr(ws), wsb, stream())
    return to_np(Y), to_np(dX), to_np(dw), to_np(dc)


def _key(x):
    u = x.view(np.uint16).astype(np.int32)
    return np.where(u & 0x8000, -(u & 0x7fff), u)


@pytest.mark.parametrize("shape", [(1, 16), (50, 48), (272, 400), (1000, 768), (512, 1024), (131, 2064), (64, 4096), (140001, 16)])
@pytest.mark.parametrize("eps", [0.0, 1e-5])
def test_forward_and_backward_against_the_oracle(shape, eps):
    """Row lengths below, at and across the 512-element wave chunk; row counts that are not multiples of the
    32-row blocks of the backward pass.  FP32 statistics against double: at most one FP16 step, rarely."""
    b, n = shape
    X, w, c, G = _inputs(b, n, 181 + n, sigma=1.7, shift=0.4)
    if n == 16 and eps == 0.0:
        X[0, :] = np.arange(16, dtype=np.float16)             # a row that certainly has spread
    Y, dX, dw, dc = _run(X, w, c, G, eps)
    rY, _, _ = O.layer_norm_fwd(X, w, c, eps)
    rdX, rdw, rdc = O.layer_norm_bwd(X, w, G, eps)
    assert int(np.max(np.abs(_key(Y) - _key(rY)))) <= 1 and np.mean(Y != rY) < 5e-3
    assert_close(dX, rdX, "dX")
    assert np.mean(dX != rdX) < 0.02
    assert_close(dw, rdw, "dw")
    assert_close(dc, rdc, "dc")


def test_bert_large_shape_variances_and_determinism():
    """b = 8192 tokens, n = 1024: unit weights, N(0,1) input and gradient.  Var(Y) = 1, Var(dX) = 1 - 2/n,
    Var(dw) = Var(dc) = 1 with the default b^-1/2; two runs are bit-identical (ordered block sums)."""
    b, n = 8192, 1024
    X, _, _, G = _inputs(b, n, 191)
    one, zero = np.ones(n, np.float16), np.zeros(n, np.float16)
    Y, dX, dw, dc = _run(X, one, zero, G, 0.0)
    v = lambda a: float(np.var(a.astype(np.float64)))
    assert abs(v(Y) - 1.0) < 0.01 and abs(v(dX) - (1 - 2 / n)) < 0.01
    assert abs(v(dw) - 1.0) < 0.12 and abs(v(dc) - 1.0) < 0.12
    rows = [0, 31, 32, 4095, 8191]
    rY, _, _ = O.layer_norm_fwd(X[rows], one, zero)
    assert int(np.max(np.abs(_key(Y[rows]) - _key(rY)))) <= 1
    cols = slice(0, 64)
    _, rdw, rdc = O.layer_norm_bwd(np.ascontiguousarray(X), one, G)
    assert_close(dw, rdw, "dw") and assert_close(dc, rdc, "dc")
    Y2, dX2, dw2, dc2 = _run(X, one, zero, G, 0.0)
    assert np.array_equal(dw, dw2) and np.array_equal(dc, dc2) and np.array_equal(dX, dX2)
    # an explicit weight-gradient scale
    _, _, dw3, _ = _run(X, one, zero, G, 0.0, beta=0.5)
    assert_close(dw3, O.layer_norm_bwd(X, one, G, 0.0, 0.5)[1], "dw, beta given")


def test_zero_variance_row_and_empty_input():
    X = np.full((4, 32), 3.0, np.float16)
    X[1] = np.arange(32, dtype=np.float16)
    w, c, G = np.ones(32, np.float16), np.full(32, 0.5, np.float16), np.ones((4, 32), np.float16)
    Y, _, _, _ = _run(X, w, c, G, 0.0)
    assert np.isnan(Y[0].astype(np.float32)).all() and np.isfinite(Y[1].astype(np.float32)).all()     # 0 * inf, as the formula says
    Y, _, _, _ = _run(X, w, c, G, 1e-5)
    assert np.all(Y[0] == np.float16(0.5))
    us.layer_norm_fwd(None, None, None, None, 0, 32, 0.0, stream())
