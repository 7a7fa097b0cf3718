"""GPU parity over a seeded sweep of shapes placed around the limits where the library changes kernel, tile shape or
launch form (register-staged / direct loads, 128 x 128 / 256 x 256 / wave-split tiles, K slices, paired backward
launch), with ragged edges, and over 24 seeded random shapes.  Forward (plain, GELU, residual, with and without bias and workspace) and backward
(grad_X and grad_W in one call, with and without GELU'), FP16 and FP8, against the oracle on sampled rows."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2303_11257_amd as us
import synth
from gpu_util import DEV, assert_close, cast_fp8, empty, ptr, stream, to_dev, to_np

pytestmark = pytest.mark.gpu

# (b, m, n): what the shape is near
BASE = [
    (80, 48, 112),        # everything smaller than one tile; reduction not a multiple of a stage
    (400, 208, 272),      # register-staged kernel, several ragged tiles
    (528, 384, 400),      # direct loads, 128 x 128 tiles with ragged edges
    (1024, 1024, 2000),   # forward: at most one small tile per CU and a long reduction (wave-split small tile)
    (1040, 2048, 1008),   # the same for grad_X; grad_W cut into K slices
    (1024, 2000, 1552),   # grad_W: 208 small tiles, long reduction: wave-split tile with ragged edges
    (2048, 1792, 1536),   # grad_W: 168 tiles, in the lower part of the wave-split range
    (6000, 128, 4000),    # forward: 384 large tiles with ragged edges, one stage of reduction
    (6144, 4096, 768),    # backward of one layer in one launch (large-tile grad_X, wave-split grad_W)
    (4096, 768, 2048),    # forward and grad_X on 256 x 128 / 128 x 128 tiles, grad_W on 96 tiles (K slices)
    (6000, 2048, 1008),   # forward: 192 tiles of 256 x 128 with two wave groups, ragged in both dimensions
    (2304, 4000, 1024),   # paired backward with grad_W on 128 long (256 x 128) tiles, ragged; grad_X on 256 x 128 tiles
    (7936, 1008, 4096),   # paired backward as one round: 124 large grad_X tiles + 128 long grad_W tiles, both ragged
    (4000, 192, 3072),    # forward (FP16): 16 x 16 tiles of 256 x 192, the last row of tiles ragged
    (4096, 752, 3072),    # paired backward as one round: 96 grad_X tiles of 256 x 128 (ragged) + 144 wave-split grad_W tiles
    (4096, 3056, 768),    # paired backward: GELU' on 128 x 256 tiles (ragged) next to 144 grad_W tiles
]


def _shapes():
    rng = np.random.default_rng(20230316)
    out = []
    for b, m, n in BASE:
        out.append((b, m, n))
        jitter = lambda v: int(max(16, v + 16 * rng.integers(-2, 3)))
        out.append((jitter(b), jitter(m), jitter(n)))
    # ... and shapes nobody chose: every dimension a seeded draw, half of them multiples of 128 or 192 (so that the
    # direct-to-LDS kernels and their tile choices are reached), the rest multiples of 16 (ragged tiles, staged kernel)
    rng = np.random.default_rng(20230317)

    def draw(lo, hi):
        kind = rng.integers(0, 4)
        unit = (16, 16, 128, 192)[kind]
        return int(unit * rng.integers(max(1, lo // unit), hi // unit + 1))
    for _ in range(24):
        out.append((draw(256, 6144), draw(128, 4224), draw(128, 4224)))
    return out


def _sample(rng, extent, k=6):
    idx = {0, extent - 1}
    while len(idx) < min(k, extent):
        idx.add(int(rng.integers(0, extent)))
    return np.array(sorted(idx))


@pytest.mark.parametrize("fp8", [False, True])
@pytest.mark.parametrize("shape", _shapes())
def test_forward_and_backward(shape, fp8):
    b, m, n = shape
    rng = np.random.default_rng(b * 7 + m * 3 + n)
    X, W, G = synth.linear_inputs(b, m, n, 300 + b + m + n)
    bias = synth.normal(301, 9, (n,), sigma=0.5)
    skip = synth.normal(302, 10, (b, n))
    if fp8:
        X, W, G = cast_fp8(X, us.E4M3), cast_fp8(W, us.E4M3), cast_fp8(G, us.E5M2)
        gd, od = (us.E4M3, us.E4M3, us.E5M2), (O.E4M3, O.E4M3, O.E5M2)
    else:
        gd, od = (us.F16,) * 3, (O.F16,) * 3
    a, bx, bw = O.linear_scales(b, m, n)
    ag, bg = O.gelu_scales()
    tX, tW, tG, tb, tskip = to_dev(X), to_dev(W), to_dev(G), to_dev(bias), to_dev(skip)
    wsb = max(us.workspace_bytes(b, m, n), us.TABLE_AREA_BYTES)
    ws = torch.full((wsb,), 0x5A, dtype=torch.uint8, device=DEV)
    st = stream()
    rows = _sample(rng, b)
    ridx = torch.as_tensor(rows, device=DEV)
    Xr, Gr = X[rows], G[rows]

    # forward: plain with bias, GELU (with workspace: table path where it applies) without bias, residual with bias
    Y, Z, H16, Out = (empty((b, n), np.float16) for _ in range(4))
    H8 = empty((b, n), np.uint8)
    us.linear_bias_fwd(ptr(tX), ptr(tW), ptr(tb), ptr(Y), b, m, n, gd[0], gd[1], us.F16, 0.0, us.EPI_NONE, 0.0, None, None, None, 0, st)
    us.linear_fwd(ptr(tX), ptr(tW), ptr(Z), b, m, n, gd[0], gd[1], us.F16, 0.0, us.EPI_GELU, 0.0, ptr(H16), ptr(H8) if fp8 else None,
                  ptr(ws), wsb, st)
    us.linear_bias_fwd(ptr(tX), ptr(tW), ptr(tb), ptr(Out), b, m, n, gd[0], gd[1], us.F16, 0.0, us.EPI_RESIDUAL, 0.6, ptr(tskip), None,
                       None, 0, st)
    torch.cuda.synchronize()
    Yref = O.linear_fwd(Xr, W, a, od[0], od[1], bias=bias)
    assert_close(Y[ridx].cpu().numpy(), Yref, "Y + bias", fp8=fp8)
    Zr = Z[ridx].cpu().numpy()
    assert_close(Zr, O.linear_fwd(Xr, W, a, od[0], od[1]), "Z", fp8=fp8)
    Hr = H16[ridx].cpu().numpy()
    assert_close(Hr, O.gelu_fwd(Zr, ag), "H")
    if fp8:
        assert np.array_equal(H8[ridx].cpu().numpy(), O.cast_fp8(Hr, O.E4M3)[0])
    sw, bwt = np.float32(np.sqrt(1 - np.float32(0.6) ** 2)), np.float32(0.6)
    assert_close(Out[ridx].cpu().numpy(), O.weighted_add2(skip[rows], Y[ridx].cpu().numpy(), sw, bwt), "Out")

    # backward: grad_X and grad_W in one call, plain and with GELU' (pre-activation = a unit-scale tensor of X's shape)
    Zpre = synth.normal(303, 11, (b, m))
    tZ = to_dev(Zpre)
    dX, dXg, dW, dW2 = empty((b, m), np.float16), empty((b, m), np.float16), empty((m, n), np.float16), empty((m, n), np.float16)
    dZ8 = empty((b, m), np.uint8)
    us.linear_bwd(ptr(tX), ptr(tW), ptr(tG), ptr(dX), ptr(dW), b, m, n, *gd, us.F16, 0.0, 0.0, us.EPI_NONE, 0.0, None, None, ptr(ws), wsb, st)
    us.linear_bwd(ptr(tX), ptr(tW), ptr(tG), ptr(dXg), ptr(dW2), b, m, n, *gd, us.F16, 0.0, 0.0, us.EPI_GELU_GRAD, 0.0, ptr(tZ),
                  ptr(dZ8) if fp8 else None, ptr(ws), wsb, st)
    torch.cuda.synchronize()
    dXref = O.linear_bwd_dx(Gr, W, bx, od[2], od[1])
    assert_close(dX[ridx].cpu().numpy(), dXref, "dX", fp8=fp8)
    dXg_r = dXg[ridx].cpu().numpy()
    assert_close(dXg_r, O.gelu_bwd(Zpre[rows], dX[ridx].cpu().numpy(), bg), "dX with GELU'", fp8=fp8)   # the two grad_X launches may use different tiles
    if fp8:
        assert np.array_equal(dZ8[ridx].cpu().numpy(), O.cast_fp8(dXg_r, O.E5M2)[0])
    wr = _sample(rng, m)                      # rows of dW = columns of X
    widx = torch.as_tensor(wr, device=DEV)
    dWref = O.linear_bwd_dw(np.ascontiguousarray(X[:, wr]), G, bw, od[0], od[2])
    assert_close(dW[widx].cpu().numpy(), dWref, "dW", fp8=fp8)
    # grad_W has its own kernel alone and another in a paired launch (whether a pair forms depends on grad_X's epilogue
    # too): the same sum added in another order, so nearly every FP16 result is the same and the rest a rounding apart
    assert_close(dW2[widx].cpu().numpy(), dWref, "dW next to GELU'", fp8=fp8)
    assert (dW != dW2).float().mean().item() < 0.2
