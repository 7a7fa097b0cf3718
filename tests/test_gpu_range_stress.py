"""GPU parity for the FP8 range-stress sweep: a scaled cast to E4M3 followed by a matmul on the cast operands.

Square products M = N = K in {2048, 4096, 8192}; X and W are N(0, sigma^2) in FP32, sigma in {1/64, 1/8, 1, 8, 64}, with
one entry in 1000 replaced by +-1000 (the outlier model of App. D).  Each run casts both operands with scale s (s = 1: a
mis-scaled tensor clips at +-448 or falls into the subnormals and below; s = 1/sigma: the per-tensor scaling that unit
scaling makes unnecessary), checks the codes bit for bit and the four counters (clipping and underflow, Sec. 3.1
"Quantisation error") against the oracle, then multiplies the codes with alpha = K^-1/2 / (s_x s_w) and compares the FP16
result with the oracle's product of the GPU's own codes on a slab of 256 rows and on sampled columns.

Two bounds on the product, with S the RMS of the reference (these outputs are not unit-scale) and
B[i,j] = alpha * sum_k |x_ik| |w_kj| (the oracle's product of the codes with their sign bits cleared):
  * always required:  |gpu - ref| <= 2e-3 * max(|ref|, S) + 2e-4 * S + 2^-12 * B.  The last term is the forward error of
    a sum whose adder keeps about 14 bits below the largest product of a group (measured on this matrix core): it is
    what lets an output pass in which two outlier products, 448 x 448 each, cancel (|ref| small, the error set by the
    products that were dropped beside them);
  * the bound of the unit-scaled tensors (floor S / 64, no B term): met by the runs whose operands have a narrow range
    (sigma = 64 cast with s = 1, where the clipped outliers are 7 sigma; sigma = 1/64 with s = 1, where everything but
    the outliers is negligible), NOT met where codes of magnitude 100 ... 448 sit among unit-scale codes: every product
    that shares an adder group with an outlier's loses its low bits.  The error of an output near zero is then up to
    4e-3 of the outputs' bulk scale (40 times what N(0,1) operands show) and 1 % of it where two outlier products
    cancel; the vendor library's kernel gives the same figures to three digits on the same codes.  Such a run is
    reported as an expected failure with its measured figure, not hidden by a wider bound."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2303_11257_amd as us
import synth
from gpu_util import DEV, RTOL, assert_close, empty, ptr, rel_err, stream

pytestmark = pytest.mark.gpu

_BASE = {}


def _oracle_cast(a, fmt, scale, workers=16):
    """The oracle's cast on slices of the tensor in parallel (it is elementwise and serial; 67 M elements take it 5 s):
    codes concatenated, counters added."""
    import concurrent.futures
    flat = a.reshape(-1)
    bounds = [int(v) for v in np.linspace(0, flat.size, workers + 1)]
    with concurrent.futures.ThreadPoolExecutor(workers) as ex:
        res = list(ex.map(lambda lo_hi: O.cast_fp8(flat[lo_hi[0]:lo_hi[1]], fmt, scale), zip(bounds[:-1], bounds[1:])))
    codes = np.concatenate([r[0] for r in res]).reshape(a.shape)
    stats = {k: sum(r[1][k] for r in res) for k in O.STAT_NAMES}
    return codes, stats


def _draws(N):
    """FP32 N(0,1) draws and outlier positions of the two operands at size N (once per size: drawing 2 x 67 M normals
    takes seconds; every sigma reuses them, which for sigma a power of two is exactly what a fresh draw would give)."""
    if N not in _BASE:
        _BASE.clear()                                         # one size at a time in memory
        seed = synth.C4_SEED + N
        _BASE[N] = tuple((synth.normal(seed, t, (N, N), 1.0, np.float32), synth.outlier_positions(seed, t, N * N))
                         for t in (synth.T_X, synth.T_W1))
    return _BASE[N]


def _cases():
    out = []
    for N in synth.C4_SIZES:
        for sigma in synth.C4_SIGMAS:
            for per_tensor in (False, True):
                if per_tensor and sigma == 1.0:
                    continue                                  # s = 1/sigma = 1: the same run
                out.append((N, sigma, per_tensor))
    return out


@pytest.mark.parametrize("N,sigma,per_tensor", _cases(), ids=lambda v: str(v))
def test_scaled_cast_then_matmul(N, sigma, per_tensor, record_property):
    (bx, px), (bw, pw) = _draws(N)
    s = float(1.0 / sigma) if per_tensor else 1.0
    st = stream()
    codes, host = [], []
    for base, pos in ((bx, px), (bw, pw)):
        a = synth.place_outliers(base, sigma, pos)
        src = torch.from_numpy(a).to(DEV)
        dst = empty((N, N), np.uint8)
        stats = torch.zeros(4, dtype=torch.int64, device=DEV)
        us.cast_fp8(ptr(src), us.F32, ptr(dst), us.E4M3, N * N, s, ptr(stats), st)
        torch.cuda.synchronize()
        ref_codes, ref_stats = _oracle_cast(a, O.E4M3, s)
        got = dst.cpu().numpy()
        assert np.array_equal(got, ref_codes), "E4M3 codes differ from the oracle"
        got_stats = dict(zip(O.STAT_NAMES, (int(v) for v in stats.cpu().numpy())))
        assert got_stats == ref_stats, (got_stats, ref_stats)
        # the outliers, and only they, clip whenever 1000 s > 448 (7 sigma s stays below 448 for every sigma here)
        if 1000.0 * s > 448.0:
            assert ref_stats["n_sat"] == pos[0].size
        assert ref_stats["n_nan"] == 0
        codes.append(dst)
        host.append(got)
        del src, a
    X8, W8 = codes
    Y = empty((N, N), np.float16)
    alpha = float(np.float32(N ** -0.5) / np.float32(s * s))
    us.linear_fwd(ptr(X8), ptr(W8), ptr(Y), N, N, N, us.E4M3, us.E4M3, us.F16, alpha, us.EPI_NONE, 0.0, None, None, None, 0, st)
    torch.cuda.synchronize()
    assert "direct:256x256" in us.last_launch() or N < 4096, us.last_launch()
    # oracle on the GPU's own codes: a slab of 256 consecutive rows (one row of large tiles, all columns) ...
    r0 = (N // 2 // 256) * 256
    ref = O.linear_fwd(host[0][r0:r0 + 256], host[1], alpha, O.E4M3, O.E4M3)
    fin = np.isfinite(ref.astype(np.float32))
    scale = float(np.sqrt(np.mean(ref[fin].astype(np.float64) ** 2)))          # the output's own scale
    Yr = Y[r0:r0 + 256].cpu().numpy()
    mag = [h & 0x7F for h in host]                                             # the codes of |x|, |w|
    B = O.linear_fwd(mag[0][r0:r0 + 256], mag[1], alpha, O.E4M3, O.E4M3, O.F32).astype(np.float64)
    assert_close(Yr, ref, f"Y rows (floor S, forward-error term) N={N} sigma={sigma} s={s}", fp8=True, scale=scale, tau=1.0,
                 allow=2.0 ** -12 * B)
    # ... and 32 sampled columns over all rows
    rng = np.random.default_rng(N + int(sigma * 64))
    cols = np.sort(rng.choice(N, 32, replace=False))
    refc = O.linear_fwd(host[0], np.ascontiguousarray(host[1][:, cols]), alpha, O.E4M3, O.E4M3)
    Yc = Y[:, torch.as_tensor(cols, device=DEV)].cpu().numpy()
    Bc = O.linear_fwd(mag[0], np.ascontiguousarray(mag[1][:, cols]), alpha, O.E4M3, O.E4M3, O.F32).astype(np.float64)
    assert_close(Yc, refc, f"Y columns (floor S, forward-error term) N={N} sigma={sigma} s={s}", fp8=True, scale=scale, tau=1.0,
                 allow=2.0 ** -12 * Bc)
    # what the mis-scaled cast did to the product: reported, not gated (overflow to inf is compared by class above)
    n_inf = int(torch.isinf(Y).sum().item())
    print(f"range stress N={N} sigma={sigma} s={s}: output rms {scale:.3e}, inf outputs {n_inf}")
    # the bound of the unit-scaled tensors (floor S / 64)
    tight = max(rel_err(Yr, ref, fp8=True, scale=scale), rel_err(Yc, refc, fp8=True, scale=scale))
    record_property("gated_with_floor_S_over_64", tight)
    if tight > RTOL:
        pytest.xfail(f"codes of magnitude >= 100 among unit-scale codes: the matrix core's narrow adder leaves the 2e-3 bound with "
                     f"floor S/64 (measured {tight:.2e}); within 2e-3 max(|ref|, S) + 2^-12 sum|x w|")
