"""GPU parity for the scaled sum over the last dimension (us_sum_fwd / us_sum_bwd) against the oracle."""
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


@pytest.mark.parametrize("shape", [(1, 8), (37, 72), (300, 512), (129, 1000), (65, 4096), (7, 40000), (100000, 16)])
def test_sum_fwd_and_bwd(shape):
    rows, n = shape
    x = synth.normal(121, 1, shape)
    g = synth.normal(121, 2, (rows,))
    tx, ty = to_dev(x), empty((rows,), np.float16)
    us.sum_fwd(ptr(tx), ptr(ty), rows, n, 0.0, stream())
    y, ref = to_np(ty), O.sum_fwd(x)
    # FP32 partial sums per lane, then the butterfly, against a double sum: one FP16 step at a rounding boundary, plus the
    # absolute error of the FP32 additions where a sum cancels
    assert np.all(np.abs(y.astype(np.float64) - ref.astype(np.float64)) <= 2.0 ** -10 * np.abs(ref.astype(np.float64)) + 1e-5)
    tg, td = to_dev(g), empty((rows, n), np.float16)
    us.sum_bwd(ptr(tg), ptr(td), rows, n, 0.0, stream())
    assert np.array_equal(_bits(to_np(td)), _bits(O.sum_bwd(g, n)))
    us.sum_bwd(ptr(tg), ptr(td), rows, n, 0.375, stream())
    assert np.array_equal(_bits(to_np(td)), _bits(O.sum_bwd(g, n, beta=0.375)))


def test_sum_exact_integers_and_empty_rows():
    x = synth.small_ints(122, 1, (64, 1040))
    tx, ty = to_dev(x), empty((64,), np.float16)
    us.sum_fwd(ptr(tx), ptr(ty), 64, 1040, 2.0 ** -4, stream())
    assert np.array_equal(_bits(to_np(ty)), _bits(O.sum_fwd(x, alpha=2.0 ** -4)))
    ty = torch.full((5,), 3.0, dtype=torch.float16, device=DEV)
    us.sum_fwd(None, ptr(ty), 5, 0, 0.0, stream())
    assert not to_np(ty).any()


def test_sum_propagates_nan_and_infinity():
    x = synth.normal(123, 1, (4, 64))
    x[1, 9] = np.nan
    x[2, 3] = np.inf
    x[3, 3] = np.inf; x[3, 40] = -np.inf
    tx, ty = to_dev(x), empty((4,), np.float16)
    us.sum_fwd(ptr(tx), ptr(ty), 4, 64, 0.0, stream())
    y = to_np(ty)
    assert np.isfinite(y[0]) and np.isnan(y[1]) and np.isposinf(y[2]) and np.isnan(y[3])
    ref = O.sum_fwd(x)
    assert np.array_equal(np.isnan(y), np.isnan(ref)) and np.array_equal(np.isinf(y), np.isinf(ref))
