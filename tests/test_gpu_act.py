"""GPU parity: relu / tanh / sigmoid, stand-alone and fused into the matmul epilogues (Table A.2, App. H)."""
import numpy as np
import pytest

import oracle
import paper_2303_11257_amd as us
import synth
from gpu_util import assert_close, cast_fp8, empty, linear_bwd, linear_fwd, ptr, stream, to_dev, to_np

pytestmark = pytest.mark.gpu
O = oracle
KINDS = [(us.ACT_GELU, O.GELU), (us.ACT_RELU, O.RELU), (us.ACT_TANH, O.TANH), (us.ACT_SIGMOID, O.SIGMOID)]


def _key(x):
    u = x.view(np.uint16).astype(np.int32)
    return np.where(u & 0x8000, -(u & 0x7fff), u)


def _ulps(a, b):
    fin = np.isfinite(a.astype(np.float32)) & np.isfinite(b.astype(np.float32))
    assert np.array_equal(np.isnan(a.astype(np.float32)), np.isnan(b.astype(np.float32)))
    assert np.array_equal(a[np.isinf(a.astype(np.float32))], b[np.isinf(b.astype(np.float32))])
    return int(np.max(np.abs(_key(a[fin]) - _key(b[fin]))))


@pytest.mark.parametrize("gk,ok", KINDS)
def test_every_fp16_input(gk, ok):
    """All 65536 FP16 bit patterns, default unit-scaling factors: at most one FP16 step from the oracle
    (the GPU evaluates in FP32 with exp2 / reciprocal approximations), equal almost everywhere."""
    z = np.arange(65536, dtype=np.uint32).astype(np.uint16).view(np.float16)
    a, b = O.act_scales(ok)
    tz, h = to_dev(z), empty(z.shape, np.float16)
    us.act_fwd(ptr(tz), ptr(h), z.size, us.F16, gk, 0.0, 0.0, stream())
    got, ref = to_np(h), O.act_fwd(z, ok, a)
    assert _ulps(got, ref) <= 1
    fin = np.isfinite(ref.astype(np.float32))
    assert np.mean(got[fin] != ref[fin]) < 0.02
    gh = synth.normal(167, 3, z.shape)
    tg, gz = to_dev(gh), empty(z.shape, np.float16)
    us.act_bwd(ptr(tz), ptr(tg), ptr(gz), z.size, us.F16, gk, 0.0, 0.0, stream())
    got, ref = to_np(gz), O.act_bwd(z, gh, ok, b)
    fin = np.isfinite(ref.astype(np.float32))
    if ok == O.GELU:
        # gelu' of a negative argument is formed as beta - beta*gelu'(|z|) (one table serves both signs): accurate to
        # 1e-7 absolutely, not relatively, where the slope is nearly zero
        assert_close(np.where(fin, got, 0), np.where(fin, ref, 0), "gelu bwd")
    else:
        assert _ulps(got, ref) <= 1
    assert np.mean(got[fin] != ref[fin]) < 0.02


@pytest.mark.parametrize("gk,ok", KINDS[1:])
def test_aligned_form_fp32_and_ragged_length(gk, ok):
    """f(s1 x) s2 with explicit factors, FP32 storage, a length that is not a multiple of the vector width."""
    n = 100_003
    z = synth.normal(173, 1, (n,), sigma=2.0).astype(np.float32)
    gh = synth.normal(173, 2, (n,)).astype(np.float32)
    s1, s2 = 0.75, 2.5
    tz, tg, out = to_dev(z), to_dev(gh), empty((n,), np.float32)
    us.act_fwd(ptr(tz), ptr(out), n, us.F32, gk, s1, s2, stream())
    ref = O.act_fwd(z, ok, s2, s1)
    assert np.max(np.abs(to_np(out) - ref) / np.maximum(np.abs(ref), 1e-6)) < 5e-6
    us.act_bwd(ptr(tz), ptr(tg), ptr(out), n, us.F32, gk, s1, s2, stream())
    ref = O.act_bwd(z, gh, ok, s2, s1)
    assert np.max(np.abs(to_np(out) - ref) / np.maximum(np.abs(ref), 1e-6)) < 5e-6
    us.act_fwd(None, None, 0, us.F16, gk, 0.0, 0.0, stream())          # empty input


@pytest.mark.parametrize("fp8", [False, True])
@pytest.mark.parametrize("gk,ok,flag", [(us.ACT_RELU, O.RELU, us.EPI_ACT_RELU), (us.ACT_TANH, O.TANH, us.EPI_ACT_TANH),
                                        (us.ACT_SIGMOID, O.SIGMOID, us.EPI_ACT_SIGMOID)])
@pytest.mark.parametrize("shape", [(272, 144, 400), (2048, 256, 2048)])
def test_fused_activation_epilogues(fp8, gk, ok, flag, shape):
    """Linear + activation and grad_X + activation' in one kernel, stage-wise against the oracle: the activation is
    checked on the GPU's own stored FP16 matmul result; the FP8 copies are bit-exact casts of the stored FP16 values."""
    b, m, n = shape
    X, W, G = synth.linear_inputs(b, m, n, 179)
    if fp8:
        Xo, Wo, Go = cast_fp8(X, us.E4M3), cast_fp8(W, us.E4M3), cast_fp8(G, us.E5M2)
        gdt, odt = (us.E4M3, us.E4M3, us.E5M2), (O.E4M3, O.E4M3, O.E5M2)
    else:
        Xo, Wo, Go, gdt, odt = X, W, G, (us.F16,) * 3, (O.F16,) * 3
    a, bsc = O.act_scales(ok)
    Z, H16, H8 = linear_fwd(Xo, Wo, gdt[0], gdt[1], epi=us.EPI_GELU | flag, want16=True, want8=True,
                            workspace_bytes=us.workspace_bytes(b, m, n))          # a workspace must not switch on gelu's table
    assert_close(Z, O.linear_fwd(Xo, Wo, m ** -0.5, odt[0], odt[1]), "Z", fp8=fp8)
    ref = O.act_fwd(Z, ok, a)
    assert _ulps(H16, ref) <= 1 and np.mean(H16 != ref) < 0.02
    assert np.array_equal(H8, O.cast_fp8(H16, O.E4M3)[0])
    Zpre = synth.normal(179, 7, (b, m))
    dH, _, _ = linear_bwd(None, Wo, Go, *gdt, do_dw=False)
    dZ, _, dZ8 = linear_bwd(None, Wo, Go, *gdt, epi=us.EPI_GELU_GRAD | flag, Zpre=Zpre, want8=True, do_dw=False)
    # (the plain and the fused grad_X may come from different tile shapes, i.e. other summation orders: dH agrees to
    # the matmul tolerance, not to the bit, so the product is compared the same way)
    ref = O.act_bwd(Zpre, dH, ok, bsc)
    assert_close(dZ, ref, "dZ", fp8=fp8)
    assert np.mean(dZ != ref) < 0.05
    assert np.array_equal(dZ8, O.cast_fp8(dZ, O.E5M2)[0])
    # variance: unit after the scaled activation, forward and backward
    if b >= 2048:
        assert abs(np.std(H16.astype(np.float64)) - 1.0) < 0.03
        assert abs(np.sqrt(np.mean(dZ.astype(np.float64) ** 2)) - 1.0) < 0.03
