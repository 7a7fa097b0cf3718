"""GPU parity for the scaled softmax (forward / backward) and the softmax cross-entropy against the oracle."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2303_11257_amd as us
import synth
from gpu_util import DEV, empty, ptr, stream, to_dev, to_np

pytestmark = pytest.mark.gpu


def _bits(a):
    return np.ascontiguousarray(a).view(np.uint16)


def _one_step(gpu, ref, rate=0.01):
    """FP32 exponentials and sums on the GPU, double in the oracle: the rounded FP16 results agree except where the
    value sits next to a rounding boundary (one step, in few places); near zero the step is tiny in absolute terms."""
    g, r = gpu.astype(np.float64), ref.astype(np.float64)
    assert np.array_equal(np.isnan(g), np.isnan(r))
    ok = ~np.isnan(r)
    assert np.all(np.abs(g[ok] - r[ok]) <= 2.0 ** -10 * np.abs(r[ok]) + 1e-6)
    assert np.mean(_bits(gpu)[ok] != _bits(ref)[ok]) < rate


def _softmax(x, s1=0.0, alpha=0.0):
    rows, s = x.shape
    tx, ty = to_dev(x), empty((rows, s), np.float16)
    us.softmax_fwd(ptr(tx), ptr(ty), rows, s, s1, alpha, stream())
    return to_np(ty)


def _softmax_bwd(x, g, s1=0.0, beta=0.0):
    rows, s = x.shape
    tx, tg, td = to_dev(x), to_dev(g), empty((rows, s), np.float16)
    us.softmax_bwd(ptr(tx), ptr(tg), ptr(td), rows, s, s1, beta, stream())
    return to_np(td)


# every register-chunk count (1, 2, 4, 8 chunks of 512 columns) with ragged lengths, and a single row
SHAPES = [(1, 8), (37, 72), (301, 128), (1000, 512), (515, 520), (333, 1000), (129, 2048), (67, 3000), (40, 4096)]


@pytest.mark.parametrize("shape", SHAPES)
def test_softmax_fwd_and_bwd(shape):
    rows, s = shape
    x = synth.normal(91, 1, shape, sigma=1.5)
    g = synth.normal(91, 2, shape)
    _one_step(_softmax(x), O.softmax_fwd(x))
    _one_step(_softmax_bwd(x, g), O.softmax_bwd(x, g))


def test_softmax_explicit_factors_and_temperature():
    x = synth.normal(92, 1, (200, 384), sigma=3.0)
    g = synth.normal(92, 2, (200, 384))
    _one_step(_softmax(x, s1=0.25, alpha=1.0), O.softmax_fwd(x, alpha=1.0, s1=0.25))
    _one_step(_softmax_bwd(x, g, s1=0.25, beta=7.0), O.softmax_bwd(x, g, beta=7.0, s1=0.25))


def test_softmax_special_rows():
    s = 64
    x = np.zeros((6, s), np.float16)
    x[1] = 11.0                                       # constant rows: exactly alpha / s = 1
    x[2, 5] = np.nan                                  # NaN anywhere: the whole row
    x[3, :] = 60000.0; x[3, 7] = -60000.0             # large finite values: the maximum is subtracted
    x[4, 9] = np.inf                                  # +inf: inf - inf in that place, NaN row
    x[5, :] = -np.inf; x[5, 3] = 0.0                  # -inf entries are zeros of the softmax
    y = _softmax(x)
    ref = O.softmax_fwd(x)
    assert np.all(y[0] == 1.0) and np.all(y[1] == 1.0)
    assert np.array_equal(np.isnan(y), np.isnan(ref)) and np.all(np.isnan(y[2])) and np.all(np.isnan(y[4]))
    ok = ~np.isnan(ref)
    assert np.array_equal(_bits(y)[ok], _bits(ref)[ok])
    assert y[5, 3] == s and y[5].astype(np.float64).sum() == s


def test_softmax_at_attention_size_sampled():
    rows, s = 16 * 16 * 512, 512                      # 16 sequences x 16 heads x 512 queries, 512 keys
    tx = synth.normal_on_device(20230314, 1, (rows, s))
    tg = synth.normal_on_device(20230314, 2, (rows, s))
    ty, td = torch.empty_like(tx), torch.empty_like(tx)
    us.softmax_fwd(ptr(tx), ptr(ty), rows, s, 0.0, 0.0, stream())
    us.softmax_bwd(ptr(tx), ptr(tg), ptr(td), rows, s, 0.0, 0.0, stream())
    torch.cuda.synchronize()
    idx = torch.as_tensor(np.array([0, 1, 63, 64, 4097, 70001, rows - 1]), device=DEV)
    x, g = tx[idx].cpu().numpy(), tg[idx].cpu().numpy()
    _one_step(ty[idx].cpu().numpy(), O.softmax_fwd(x), rate=0.02)
    _one_step(td[idx].cpu().numpy(), O.softmax_bwd(x, g), rate=0.02)
    assert abs(float(ty.float().mean()) - 1.0) < 1e-3                      # about a vector of ones
    assert abs(float(td.float().std()) - np.sqrt(np.e)) < 0.1              # see the oracle's pin for the factor


def _xent(x, t, s1=0.0, beta=0.0, want_loss=True, want_dx=True):
    rows, s = x.shape
    tx, tt = to_dev(x), torch.from_numpy(np.ascontiguousarray(t, dtype=np.int32)).to(DEV)
    loss = torch.full((rows,), -7.0, dtype=torch.float32, device=DEV) if want_loss else None
    dx = empty((rows, s), np.float16) if want_dx else None
    us.softmax_xent(ptr(tx), ptr(tt), ptr(loss), ptr(dx), rows, s, s1, beta, stream())
    torch.cuda.synchronize()
    return (loss.cpu().numpy() if want_loss else None), (to_np(dx) if want_dx else None)


@pytest.mark.parametrize("shape", [(5, 8), (64, 256), (33, 1000), (19, 30528), (3, 65536)])
def test_xent_against_the_oracle(shape):
    rows, s = shape
    x = synth.normal(93, 1, shape, sigma=2.0)
    t = (np.arange(rows) * 7919 + 3) % s
    if rows > 4:
        t[2], t[4] = -1, s                              # rows without a label
    loss, dx = _xent(x, t)
    rl, rd = O.softmax_xent(x, t)
    assert np.allclose(loss, rl, rtol=2e-6, atol=2e-6)
    _one_step(dx, rd)
    if rows > 4:
        assert loss[2] == 0 and loss[4] == 0 and not dx[2].any() and not dx[4].any()
    # either output alone
    l2, _ = _xent(x, t, want_dx=False)
    _, d2 = _xent(x, t, want_loss=False)
    assert np.array_equal(l2, loss) and np.array_equal(_bits(d2), _bits(dx))


def test_xent_factors_and_the_uniform_case_of_app_g():
    s = 1024
    x = np.zeros((4, s), np.float16)
    t = np.array([0, 1, 500, 1023])
    loss, dx = _xent(x, t)
    assert np.allclose(loss, np.log(s), rtol=1e-6)
    d = dx.astype(np.float64)
    assert np.all(np.abs((d ** 2).mean(axis=1) - 1.0) < 2e-3) and np.all(np.abs(d.mean(axis=1)) < 1e-3)   # beta = s / sqrt(s-1): unit variance
    x = synth.normal(94, 1, (16, 640), sigma=2.0)
    t = np.arange(16) * 37 % 640
    loss, dx = _xent(x, t, s1=0.5, beta=3.0)
    rl, rd = O.softmax_xent(x, t, beta=3.0, s1=0.5)
    assert np.allclose(loss, rl, rtol=2e-6, atol=2e-6)
    _one_step(dx, rd)
