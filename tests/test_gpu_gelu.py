"""GPU parity: stand-alone unit-scaled GELU forward / backward against the oracle."""
import numpy as np
import pytest

import oracle
import paper_2303_11257_amd as us
import synth
from gpu_util import assert_close, empty, ptr, stream, to_dev, to_np

pytestmark = pytest.mark.gpu


def _run_fwd(z, alpha=0.0):
    tz = to_dev(z.reshape(-1))
    th = empty((z.size,), z.dtype)
    us.gelu_fwd(ptr(tz), ptr(th), z.size, us.F16 if z.dtype == np.float16 else us.F32, alpha, stream())
    return to_np(th).reshape(z.shape)


def _run_bwd(z, g, beta=0.0):
    tz, tg = to_dev(z.reshape(-1)), to_dev(g.reshape(-1))
    to = empty((z.size,), z.dtype)
    us.gelu_bwd(ptr(tz), ptr(tg), ptr(to), z.size, us.F16 if z.dtype == np.float16 else us.F32, beta, stream())
    return to_np(to).reshape(z.shape)


def test_fwd_every_fp16_input():
    h = np.arange(65536, dtype=np.uint32).astype(np.uint16).view(np.float16)
    h = h[np.isfinite(h.astype(np.float32))]
    ag, _ = oracle.gelu_scales()
    got = _run_fwd(h)                       # default scale = the unit-scaling factor
    want = oracle.gelu_fwd(h, ag)
    assert_close(got, want, "gelu fwd")
    ulp = np.abs(got.view(np.uint16).astype(np.int32) - want.view(np.uint16).astype(np.int32))
    assert ulp.max() <= 1 and np.mean(ulp != 0) < 0.01     # FP32 evaluation may flip an FP16 tie
    assert np.array_equal(_run_fwd(h, float(ag)), got)


def test_bwd_every_fp16_z_with_random_gradient():
    h = np.arange(65536, dtype=np.uint32).astype(np.uint16).view(np.float16)
    h = h[np.isfinite(h.astype(np.float32))]
    g = synth.normal(79, 2, h.shape)
    _, bg = oracle.gelu_scales()
    got = _run_bwd(h, g)
    want = oracle.gelu_bwd(h, g, bg)
    assert_close(got, want, "gelu bwd")
    d = np.abs(got.astype(np.float64) - want.astype(np.float64))
    assert d.max() < 2e-3 * np.abs(g.astype(np.float64)).max()


@pytest.mark.parametrize("n", [1, 7, 8, 9, 1001, 1 << 20])
@pytest.mark.parametrize("dtype", [np.float16, np.float32])
def test_ragged_lengths_and_fp32(n, dtype):
    z = synth.normal(83, 1, (n,), sigma=1.5, dtype=dtype)
    g = synth.normal(83, 2, (n,), dtype=dtype)
    ag, bg = oracle.gelu_scales()
    assert_close(_run_fwd(z), oracle.gelu_fwd(z, ag), "fwd")
    assert_close(_run_bwd(z, g), oracle.gelu_bwd(z, g, bg), "bwd")
    if dtype == np.float32:
        assert np.max(np.abs(_run_fwd(z).astype(np.float64) - oracle.gelu_fwd(z, ag).astype(np.float64))) < 1e-5


def test_in_place_and_custom_scale():
    z = synth.normal(89, 1, (4096,))
    tz = to_dev(z)
    us.gelu_fwd(ptr(tz), ptr(tz), z.size, us.F16, 1.0, stream())
    assert_close(to_np(tz), oracle.gelu_fwd(z, 1.0), "in-place")


def test_unit_variance_on_the_gpu():
    z = synth.normal(97, 1, (1 << 20,))
    g = synth.normal(97, 2, (1 << 20,))
    assert abs(_run_fwd(z).astype(np.float64).std() - 1.0) < 0.01
    assert abs(np.sqrt(np.mean(_run_bwd(z, g).astype(np.float64) ** 2)) - 1.0) < 0.01
