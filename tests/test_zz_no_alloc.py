"""GPU: us_linear_bwd_noalloc (static device scratch, no allocation) against us_linear_bwd given a workspace.

Both run the same kernels, so every output must be identical bit for bit.  Each case makes two calls in a row through
the C ABI, the second on a smaller input, so that whatever the first call left in the shared scratch (tables, FP32
slices of a larger grad_W) is still there when the second runs.  Collected last (file name): it must pass alone in a
fresh process and after every other test."""
import numpy as np
import pytest
import torch

import paper_2303_11257_amd as us
import synth
from gpu_util import DEV, cast_fp8, empty, ptr, stream, to_dev

pytestmark = pytest.mark.gpu


def _run(shape, fp8, epi, seed, noalloc):
    b, m, n = shape
    X, W, G = synth.linear_inputs(b, m, n, seed)
    if fp8:
        X, W, G = cast_fp8(X, us.E4M3), cast_fp8(W, us.E4M3), cast_fp8(G, us.E5M2)
        gdt = (us.E4M3, us.E4M3, us.E5M2)
    else:
        gdt = (us.F16,) * 3
    tX, tW, tG = to_dev(X), to_dev(W), to_dev(G)
    tZ = to_dev(synth.normal(seed, 7, (b, m))) if epi else None
    dX, dW = empty((b, m), np.float16), empty((m, n), np.float16)
    dX.fill_(3.0), dW.fill_(3.0)
    a8 = torch.full((b, m), 0x55, dtype=torch.uint8, device=DEV) if (epi and fp8) else None
    st = stream()
    if noalloc:
        us.linear_bwd_noalloc(ptr(tX), ptr(tW), ptr(tG), ptr(dX), ptr(dW), b, m, n, *gdt, us.F16, 0.0, 0.0, epi, 0.0, ptr(tZ), ptr(a8), st)
    else:
        wsb = us.workspace_bytes(b, m, n)
        ws = torch.full((wsb,), 0xA5, dtype=torch.uint8, device=DEV)
        us.linear_bwd(ptr(tX), ptr(tW), ptr(tG), ptr(dX), ptr(dW), b, m, n, *gdt, us.F16, 0.0, 0.0, epi, 0.0, ptr(tZ), ptr(a8), ptr(ws), wsb, st)
    rec = us.last_launch()
    torch.cuda.synchronize()
    return dX.cpu().numpy(), dW.cpu().numpy(), (a8.cpu().numpy() if a8 is not None else None), rec


def _same(a, b, what):
    for x, y, name in zip(a[:3], b[:3], ("dX", "dW", "FP8 copy")):
        if x is None:
            assert y is None
            continue
        xb, yb = x.view(np.uint16) if x.dtype == np.float16 else x, y.view(np.uint16) if y.dtype == np.float16 else y
        assert np.array_equal(xb, yb), f"{what}: {name} differs ({a[3]} vs {b[3]})"
    assert a[3] == b[3], (a[3], b[3])


# (first call, second smaller call): grad_W cut into K slices twice (the second's slices are smaller than what the first
# left behind); the table-driven GELU' in a paired launch, then slices; slices, then the arithmetic GELU' on small tiles
PAIRS = [
    (((2048, 1024, 1008), us.EPI_NONE), ((1040, 528, 272), us.EPI_NONE)),
    (((6144, 4096, 768), us.EPI_GELU_GRAD), ((1040, 2048, 1008), us.EPI_NONE)),
    (((1040, 2048, 1008), us.EPI_NONE), ((528, 384, 400), us.EPI_GELU_GRAD)),
]


@pytest.mark.parametrize("fp8", [False, True])
@pytest.mark.parametrize("first,second", PAIRS)
def test_two_calls_in_a_row_match_the_workspace_entry_point(first, second, fp8):
    assert us.noalloc_scratch_bytes() == us.TABLE_AREA_BYTES + (16 << 20)
    want = [_run(shape, fp8, epi, 401 + k, noalloc=False) for k, (shape, epi) in enumerate((first, second))]
    got = [_run(shape, fp8, epi, 401 + k, noalloc=True) for k, (shape, epi) in enumerate((first, second))]     # back to back
    for k in range(2):
        _same(got[k], want[k], f"call {k + 1} {(first, second)[k][0]}")
    assert us.workspace_bytes(*first[0]) > us.TABLE_AREA_BYTES or first[1] == us.EPI_GELU_GRAD      # the scratch really was used


def test_a_shape_beyond_the_scratch_is_refused_before_any_launch():
    b, m, n = 4096, 512, 2048                       # 8 FP32 slices of 512 x 2048: 33.5 MB
    assert us.workspace_bytes(b, m, n) > us.noalloc_scratch_bytes()
    dX = torch.full((b, m), 3.0, dtype=torch.float16, device=DEV)
    dW = torch.full((m, n), 3.0, dtype=torch.float16, device=DEV)
    X, W, G = empty((b, m), np.float16), empty((m, n), np.float16), empty((b, n), np.float16)
    with pytest.raises(us.UsError) as e:
        us.linear_bwd_noalloc(ptr(X), ptr(W), ptr(G), ptr(dX), ptr(dW), b, m, n, us.F16, us.F16, us.F16, us.F16, 0.0, 0.0,
                              us.EPI_NONE, 0.0, None, None, stream())
    assert e.value.status == 5
    torch.cuda.synchronize()
    assert bool((dX == 3.0).all()) and bool((dW == 3.0).all())
