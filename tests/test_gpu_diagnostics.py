"""GPU parity: exponent histogram (exact counts) and SNR of a cast against the oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2303_11257_amd as us
import synth
from gpu_util import DEV, ptr, stream, to_dev

pytestmark = pytest.mark.gpu
O = oracle


def _hist(a):
    t = to_dev(a)
    h = torch.zeros(us.HIST_BINS, dtype=torch.int64, device=DEV)
    us.exponent_histogram(ptr(t), us.F16 if a.dtype == np.float16 else us.F32, a.size, ptr(h), stream())
    torch.cuda.synchronize()
    return h.cpu().numpy().astype(np.uint64)


def _snr(a, fmt, scale=1.0):
    t = to_dev(a)
    s = torch.zeros(2, dtype=torch.float64, device=DEV)
    us.cast_snr(ptr(t), us.F16 if a.dtype == np.float16 else us.F32, a.size, fmt, scale, ptr(s), stream())
    torch.cuda.synchronize()
    return tuple(s.cpu().numpy())


def test_histogram_every_fp16_pattern_and_a_ragged_fp32_tensor():
    v = np.arange(65536, dtype=np.uint32).astype(np.uint16).view(np.float16)
    assert np.array_equal(_hist(v), O.exponent_histogram(v))
    x = synth.normal_with_outliers(193, 1, (1_000_003,), sigma=1.0 / 64)[0].astype(np.float32)
    x[:7] = [0.0, -0.0, np.inf, -np.inf, np.nan, 1e-30, 3e9]
    got = _hist(x)
    assert np.array_equal(got, O.exponent_histogram(x)) and got.sum() == x.size
    # counters are added to, not overwritten
    t, h = to_dev(v), torch.ones(us.HIST_BINS, dtype=torch.int64, device=DEV)
    us.exponent_histogram(ptr(t), us.F16, v.size, ptr(h), stream())
    torch.cuda.synchronize()
    assert np.array_equal(h.cpu().numpy().astype(np.uint64), O.exponent_histogram(v) + 1)


@pytest.mark.parametrize("fmt,ofmt", [(us.E4M3, O.E4M3), (us.E5M2, O.E5M2)])
@pytest.mark.parametrize("sigma,scale", [(1.0, 1.0), (2.0 ** -7, 1.0), (64.0, 1.0), (64.0, 1.0 / 64)])
def test_snr_against_the_oracle(fmt, ofmt, sigma, scale):
    """Rounding, subnormal and clipping regimes, and the clipping case repaired by a cast scale.  The sums are
    formed in double on both sides, in different orders."""
    n = (1 << 21) + 5
    x = synth.normal(197, 1, (n,), sigma=sigma).astype(np.float32)
    got, ref = _snr(x, fmt, scale), O.cast_snr(x, ofmt, scale)
    assert abs(got[0] / ref[0] - 1) < 1e-9 and abs(got[1] / ref[1] - 1) < 1e-9
    x16 = synth.normal(197, 2, (n,), sigma=min(sigma, 8.0))
    got, ref = _snr(x16, fmt, scale), O.cast_snr(x16, ofmt, scale)
    assert abs(got[0] / ref[0] - 1) < 1e-9 and abs(got[1] / ref[1] - 1) < 1e-9


def test_snr_special_values_and_empty_input():
    x = np.array([1.0, -0.5, 448.0, 0.0, np.nan, 1000.0, -np.inf][:6], np.float32)
    got = _snr(x, us.E4M3)
    assert got == O.cast_snr(x, O.E4M3) == (1.0 + 0.25 + 448.0 ** 2 + 1e6, (1000.0 - 448.0) ** 2)
    s = torch.zeros(2, dtype=torch.float64, device=DEV)
    us.cast_snr(None, us.F32, 0, us.E4M3, 1.0, ptr(s), stream())
    h = torch.zeros(us.HIST_BINS, dtype=torch.int64, device=DEV)
    us.exponent_histogram(None, us.F16, 0, ptr(h), stream())
    torch.cuda.synchronize()
    assert s.sum().item() == 0 and h.sum().item() == 0
