"""GPU parity: us_cast_fp8 must reproduce the oracle's codes bit for bit and its counters exactly."""
import numpy as np
import pytest

import oracle
import paper_2303_11257_amd as us
import synth
from gpu_util import cast_fp8

pytestmark = pytest.mark.gpu

FMTS = [(us.E4M3, oracle.E4M3), (us.E5M2, oracle.E5M2)]


def _all_fp16(finite_only=True):
    h = np.arange(65536, dtype=np.uint32).astype(np.uint16).view(np.float16)
    return h[np.isfinite(h.astype(np.float32))] if finite_only else h


@pytest.mark.parametrize("fmt", FMTS)
@pytest.mark.parametrize("scale", [1.0, 2.0 ** -3, 2.0 ** 5, 1.0 / 3.0, 2.0 ** -12, 100.0])
def test_every_fp16_input(fmt, scale):
    h = _all_fp16()
    got, gs = cast_fp8(h, fmt[0], scale, want_stats=True)
    want, ws = oracle.cast_fp8(h, fmt[1], scale)
    assert np.array_equal(got, want)
    assert gs == ws


@pytest.mark.parametrize("fmt", FMTS)
def test_fp32_boundaries(fmt):
    """Every midpoint between adjacent FP8 values and its FP32 neighbours, the clip threshold, the
    flush threshold, infinities, signed zeros, FP32 subnormals."""
    top = 0x7E if fmt[1] == oracle.E4M3 else 0x7B
    table = oracle.decode(np.arange(0, top + 1, dtype=np.uint8), fmt[1])
    mid = ((table[:-1] + table[1:]) / 2).astype(np.float32)
    f = np.float32
    pts = np.concatenate([mid, np.nextafter(mid, f(0)), np.nextafter(mid, f(np.inf)), table.astype(f),
                          np.array([table[top], np.nextafter(f(table[top]), f(np.inf)), 1e30, np.inf, 0.0, 1e-45, 1e-39,
                                    np.nextafter(f(table[top] * 1.03125), f(np.inf))], f)])
    x = np.concatenate([pts, -pts])
    got, gs = cast_fp8(x, fmt[0], 1.0, want_stats=True)
    want, ws = oracle.cast_fp8(x, fmt[1], 1.0)
    assert np.array_equal(got, want)
    assert gs == ws
    assert got[-1] == (0x80 | top)


@pytest.mark.parametrize("fmt", FMTS)
@pytest.mark.parametrize("n", [1, 15, 16, 17, 4097, 1000003])
def test_ragged_lengths_fp32_and_fp16(fmt, n):
    for dtype in (np.float16, np.float32):
        x = synth.normal(71, 1, (n,), sigma=3.0, dtype=dtype)
        got, gs = cast_fp8(x, fmt[0], 0.5, want_stats=True)
        want, ws = oracle.cast_fp8(x, fmt[1], 0.5)
        assert np.array_equal(got, want)
        assert gs == ws


def test_nan_maps_to_nan_code_and_is_counted():
    x = np.array([np.nan, 1.0, -np.nan, np.inf] * 8, np.float32)
    for g, o in FMTS:
        got, gs = cast_fp8(x, g, 1.0, want_stats=True)
        want, ws = oracle.cast_fp8(x, o, 1.0)
        v = oracle.decode(got, o)
        assert np.array_equal(np.isnan(v), np.isnan(oracle.decode(want, o)))
        ok = ~np.isnan(v)
        assert np.array_equal(got[ok], want[ok])
        assert gs == ws and gs["n_nan"] == 16


def test_stats_accumulate_and_null_stats_is_allowed():
    import torch
    from gpu_util import DEV, ptr, stream, to_dev, to_np
    x = synth.normal(73, 1, (4096,), sigma=300.0, dtype=np.float32)
    src, dst = to_dev(x), torch.empty(4096, dtype=torch.uint8, device=DEV)
    stats = torch.zeros(4, dtype=torch.int64, device=DEV)
    for _ in range(3):
        us.cast_fp8(ptr(src), us.F32, ptr(dst), us.E4M3, 4096, 1.0, ptr(stats), stream())
    _, ws = oracle.cast_fp8(x, oracle.E4M3, 1.0)
    assert int(to_np(stats)[0]) == 3 * ws["n_sat"] and ws["n_sat"] > 0
    us.cast_fp8(ptr(src), us.F32, ptr(dst), us.E4M3, 4096, 1.0, None, stream())
    assert np.array_equal(to_np(dst), oracle.cast_fp8(x, oracle.E4M3, 1.0)[0])


@pytest.mark.parametrize("sigma", synth.C4_SIGMAS)
def test_range_stress_tensor_counters(sigma):
    """N(0, sigma^2) with 0.1 % +-1000 outliers: cast with s = 1 and with s = 1/sigma."""
    n = 1 << 22
    x, n_out = synth.normal_with_outliers(synth.C4_SEED, synth.T_X, (n,), sigma)
    for s in (1.0, 1.0 / sigma):
        got, gs = cast_fp8(x, us.E4M3, s, want_stats=True)
        want, ws = oracle.cast_fp8(x, oracle.E4M3, s)
        assert np.array_equal(got, want)
        assert gs == ws
        if 1000.0 * s > 448.0:
            assert gs["n_sat"] >= n_out


def test_batched_cast_equals_single_casts():
    """One launch for several tensors (ragged lengths, mixed formats) gives the oracle's codes for each."""
    import torch
    from gpu_util import DEV, ptr, stream, to_dev, to_np
    lens = [1 << 20, 16, 1, 0, 4096 * 16 + 5, 1023, 16384 * 16, 37]
    fmts = [us.E4M3, us.E5M2, us.E4M3, us.E5M2, us.E5M2, us.E4M3, us.E4M3, us.E5M2]
    xs = [synth.normal(149, i + 1, (n,), sigma=50.0) for i, n in enumerate(lens)]
    for x in xs:
        if x.size > 8:
            x[:8] = np.array([np.inf, -np.inf, np.nan, 0.0, -0.0, 6e-8, 65504.0, -500.0], np.float16)
    src = [to_dev(x) if x.size else None for x in xs]
    dst = [torch.full((max(n, 1),), 0xAA, dtype=torch.uint8, device=DEV) for n in lens]
    us.cast_fp8_batch([ptr(t) for t in src], [ptr(t) for t in dst], lens, fmts, stream())
    for x, d, n, f in zip(xs, dst, lens, fmts):
        got = to_np(d)[:n]
        want = O_cast(x, f)
        ok = ~np.isnan(x.astype(np.float32))
        assert np.array_equal(got[ok], want[ok])
        assert np.all((got[~ok] & 0x7F) >= (0x7F if f == us.E4M3 else 0x7D))
        if n == 0:
            assert to_np(d)[0] == 0xAA


def O_cast(x, f):
    return oracle.cast_fp8(x, oracle.E4M3 if f == us.E4M3 else oracle.E5M2)[0]
