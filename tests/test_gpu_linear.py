"""GPU parity: us_linear_fwd / us_linear_bwd against the oracle on the same stored operands."""
import numpy as np
import pytest

import oracle
import paper_2303_11257_amd as us
import synth
from gpu_util import assert_close, cast_fp8, linear_bwd, linear_fwd, rel_err

pytestmark = pytest.mark.gpu

O = oracle


def _operands(b, m, n, seed, fp8):
    X, W, G = synth.linear_inputs(b, m, n, seed)
    if not fp8:
        return (X, W, G), (us.F16, us.F16, us.F16), (O.F16, O.F16, O.F16)
    ops = (cast_fp8(X, us.E4M3), cast_fp8(W, us.E4M3), cast_fp8(G, us.E5M2))      # made by the GPU cast
    assert np.array_equal(ops[0], O.cast_fp8(X, O.E4M3)[0])
    return ops, (us.E4M3, us.E4M3, us.E5M2), (O.E4M3, O.E4M3, O.E5M2)


@pytest.mark.parametrize("fp8", [False, True])
def test_c1_linear_fwd_bwd(fp8):
    """Config 1: X[256,256], W[256,1024], G[256,1024], scales 1/16, 1/32, 1/16; variance within 5 % of 1."""
    b, m, n = 256, 256, 1024
    (X, W, G), gdt, odt = _operands(b, m, n, synth.CONFIGS["C1"]["seed"], fp8)
    a, bx, bw = us.linear_scales(b, m, n)
    assert (a, bx, bw) == (1 / 16, 1 / 32, 1 / 16)
    Y = linear_fwd(X, W, gdt[0], gdt[1])                               # default alpha = m^-1/2
    dX, dW, _ = linear_bwd(X, W, G, *gdt)
    assert_close(Y, O.linear_fwd(X, W, a, odt[0], odt[1]), "Y", fp8=fp8)
    assert_close(dX, O.linear_bwd_dx(G, W, bx, odt[2], odt[1]), "dX", fp8=fp8)
    assert_close(dW, O.linear_bwd_dw(X, G, bw, odt[0], odt[2]), "dW", fp8=fp8)
    for t in (Y, dX, dW):
        assert abs(np.var(t.astype(np.float64)) - 1.0) < 0.05


@pytest.mark.parametrize("fp8", [False, True])
@pytest.mark.parametrize("shape", [(16, 16, 16), (272, 144, 400), (48, 1040, 16), (528, 16, 272), (1040, 272, 528),
                                   (1040, 1152, 528), (528, 272, 1152)])
def test_ragged_shapes(fp8, shape):
    """Dimensions that are not multiples of any tile: several tiles plus a ragged tail in M, N and K.  The last two
    have a long reduction over few output tiles (forward resp. grad_X): the wave-split small tile with ragged edges."""
    b, m, n = shape
    (X, W, G), gdt, odt = _operands(b, m, n, 101 + b, fp8)
    a, bx, bw = us.linear_scales(b, m, n)
    assert_close(linear_fwd(X, W, gdt[0], gdt[1]), O.linear_fwd(X, W, a, odt[0], odt[1]), "Y", fp8=fp8)
    dX, dW, _ = linear_bwd(X, W, G, *gdt)
    assert_close(dX, O.linear_bwd_dx(G, W, bx, odt[2], odt[1]), "dX", fp8=fp8)
    assert_close(dW, O.linear_bwd_dw(X, G, bw, odt[0], odt[2]), "dW", fp8=fp8)


@pytest.mark.parametrize("fp8", [False, True])
def test_exact_integer_products(fp8):
    """Inputs in {-2..2} and power-of-two scales: every partial sum is an exact integer in FP32, so the
    GPU must equal the oracle exactly, for FP32 and FP16 outputs."""
    b, m, n = 272, 528, 400
    X = synth.small_ints(103, 1, (b, m))
    W = synth.small_ints(103, 2, (m, n))
    G = synth.small_ints(103, 4, (b, n))
    if fp8:
        X, W, G = cast_fp8(X, us.E4M3), cast_fp8(W, us.E4M3), cast_fp8(G, us.E5M2)
        gdt, odt = (us.E4M3, us.E4M3, us.E5M2), (O.E4M3, O.E4M3, O.E5M2)
    else:
        gdt, odt = (us.F16,) * 3, (O.F16,) * 3
    for out_g, out_o in ((us.F32, O.F32), (us.F16, O.F16)):
        Y = linear_fwd(X, W, gdt[0], gdt[1], alpha=0.25, out_dt=out_g)
        assert np.array_equal(Y, O.linear_fwd(X, W, 0.25, odt[0], odt[1], out_o))
        dX, dW, _ = linear_bwd(X, W, G, *gdt, beta_x=0.5, beta_w=0.125, out_dt=out_g)
        assert np.array_equal(dX, O.linear_bwd_dx(G, W, 0.5, odt[2], odt[1], out_o))
        assert np.array_equal(dW, O.linear_bwd_dw(X, G, 0.125, odt[0], odt[2], out_o))


def test_index_coded_operands_no_transposed_indexing():
    b, m, n = 64, 48, 80
    i, k = np.meshgrid(np.arange(b), np.arange(m), indexing="ij")
    X = (((i + 2 * k) % 5) - 2).astype(np.float16)
    perm = (np.arange(m) * 7) % m
    W = np.zeros((m, n), np.float16)
    W[np.arange(m), perm] = 1.0
    Y = linear_fwd(X, W, us.F16, us.F16, alpha=1.0, out_dt=us.F32)
    assert np.array_equal(Y[:, perm], X.astype(np.float32)) and np.all(Y[:, m:] == 0)
    ii, jj = np.meshgrid(np.arange(b), np.arange(n), indexing="ij")
    G = (((3 * ii + jj) % 5) - 2).astype(np.float16)
    dX, dW, _ = linear_bwd(X, W, G, us.F16, us.F16, us.F16, beta_x=1.0, beta_w=1.0, out_dt=us.F32)
    assert np.array_equal(dX, G[:, perm].astype(np.float32))
    assert np.array_equal(dW, (X.astype(np.float64).T @ G.astype(np.float64)).astype(np.float32))


def test_split_k_reduction_of_grad_w():
    """A long token dimension with a small output takes the sliced reduction path (workspace in use)."""
    b, m, n = 4096, 272, 144
    assert us.workspace_bytes(b, m, n) > 0
    for fp8 in (False, True):
        (X, W, G), gdt, odt = _operands(b, m, n, 107, fp8)
        _, dW, _ = linear_bwd(X, None, G, *gdt, do_dx=False)
        assert_close(dW, O.linear_bwd_dw(X, G, b ** -0.5, odt[0], odt[2]), "dW split", fp8=fp8)
        _, dW2, _ = linear_bwd(X, None, G, *gdt, do_dx=False)
        assert np.array_equal(dW, dW2)                          # run-to-run bit identical


@pytest.mark.parametrize("fp8", [False, True])
def test_grad_w_wave_split_reduction(fp8):
    """An output of 128-256 tiles of 128 x 128 with a long token dimension: two wave groups of one
    workgroup share the reduction and add up in LDS (no workspace).  Ragged in both output dimensions."""
    b, m, n = 1024, 2000, 1936                                   # 16 x 16 tiles, the last ones partial
    assert us.workspace_bytes(b, m, n) == us.TABLE_AREA_BYTES        # the table area only: no K slices
    (X, W, G), gdt, odt = _operands(b, m, n, 109, fp8)
    _, dW, _ = linear_bwd(X, None, G, *gdt, do_dx=False)
    assert_close(dW, O.linear_bwd_dw(X, G, b ** -0.5, odt[0], odt[2]), "dW wave split", fp8=fp8)
    # exact integers: both halves of every stage must land in the right sum
    Xi, Gi = synth.small_ints(113, 1, (b, m)), synth.small_ints(113, 4, (b, n))
    if fp8:
        Xi, Gi = cast_fp8(Xi, us.E4M3), cast_fp8(Gi, us.E5M2)
    for out_g, out_o in ((us.F32, O.F32), (us.F16, O.F16)):
        _, dWi, _ = linear_bwd(Xi, None, Gi, *gdt, beta_w=0.125, out_dt=out_g, do_dx=False)
        assert np.array_equal(dWi, O.linear_bwd_dw(Xi, Gi, 0.125, odt[0], odt[2], out_o))


@pytest.mark.parametrize("fp8", [False, True])
def test_fused_gelu_epilogues(fp8):
    """Stage-wise: Z vs the oracle matmul; H vs oracle GELU of the GPU's own stored Z; the FP8 copy vs the
    oracle cast of the GPU's own stored H (bit exact); the same for GELU' in the grad_X epilogue."""
    b, m, n = 272, 144, 400
    (X, W, G), gdt, odt = _operands(b, m, n, 109, fp8)
    ag, bg = O.gelu_scales()
    a, bx, _ = us.linear_scales(b, m, n)
    Z, H16, H8 = linear_fwd(X, W, gdt[0], gdt[1], epi=us.EPI_GELU, want16=True, want8=True)
    assert_close(Z, O.linear_fwd(X, W, a, odt[0], odt[1]), "Z", fp8=fp8)
    assert np.array_equal(Z, linear_fwd(X, W, gdt[0], gdt[1]))             # same Z with and without the epilogue
    assert_close(H16, O.gelu_fwd(Z, ag), "H")
    assert np.array_equal(H8, O.cast_fp8(H16, O.E4M3)[0])
    # FP8-only output (the fast path) carries the same codes
    _, none16, H8b = linear_fwd(X, W, gdt[0], gdt[1], epi=us.EPI_GELU, want16=False, want8=True)
    assert none16 is None and np.array_equal(H8b, H8)
    # grad_X with GELU': Zpre has the shape of dX, i.e. [b, m]
    Zpre = synth.normal(113, 7, (b, m))
    dH, _, _ = linear_bwd(None, W, G, *gdt, do_dw=False)
    assert_close(dH, O.linear_bwd_dx(G, W, bx, odt[2], odt[1]), "dH", fp8=fp8)
    dZ, _, dZ8 = linear_bwd(None, W, G, *gdt, epi=us.EPI_GELU_GRAD, Zpre=Zpre, want8=True, do_dw=False)
    assert_close(dZ, O.gelu_bwd(Zpre, dH, bg), "dZ")      # GELU' of the GPU's own dH: no matmul between the two
    assert np.array_equal(dZ8, O.cast_fp8(dZ, O.E5M2)[0])
    # codes only (no FP16 dZ stored): the same codes
    none16, _, dZ8b = linear_bwd(None, W, G, *gdt, epi=us.EPI_GELU_GRAD, Zpre=Zpre, want8=True, do_dw=False, store_dx=False)
    assert none16 is None and np.array_equal(dZ8b, dZ8)


def test_zero_reduction_length_writes_zeros():
    import torch
    from gpu_util import DEV, ptr, stream, to_np
    Y = torch.full((32, 48), 7.0, dtype=torch.float16, device=DEV)
    us.linear_fwd(None, None, ptr(Y), 32, 0, 48, us.F16, us.F16, us.F16, 1.0, us.EPI_NONE, 0.0, None, None, None, 0, stream())
    assert np.all(to_np(Y) == 0)


def test_subnormal_operands_are_honoured():
    """FP16 and FP8 subnormal inputs contribute their exact value (no flush to zero in the matrix core)."""
    b, m, n = 16, 16, 16
    X = np.zeros((b, m), np.float16)
    W = np.zeros((m, n), np.float16)
    X[:, 0] = np.float16(2.0 ** -24)
    W[0, :] = np.float16(1024.0)
    Y = linear_fwd(X, W, us.F16, us.F16, alpha=1.0, out_dt=us.F32)
    assert np.all(Y == np.float32(2.0 ** -14))
    X8 = np.zeros((b, m), np.uint8)
    W8 = np.zeros((m, n), np.uint8)
    X8[:, 0] = 0x01                       # E4M3 2^-9
    W8[0, :] = 0x38                       # E4M3 1.0
    Y = linear_fwd(X8, W8, us.E4M3, us.E4M3, alpha=1.0, out_dt=us.F32)
    assert np.all(Y == np.float32(2.0 ** -9))


def test_fp16_output_overflows_to_infinity():
    X = np.full((16, 16), 300.0, np.float16)
    Y = linear_fwd(X, X, us.F16, us.F16, alpha=1.0)
    assert np.all(np.isinf(Y.astype(np.float32)))
    assert rel_err(Y, O.linear_fwd(X, X, 1.0)) == 0.0


def test_table_driven_gelu_epilogues_equal_the_arithmetic_ones():
    """Large problems with a workspace take GELU / GELU' from a table over the FP16 pre-activation;
    the results must be bit-identical to the arithmetic epilogue (no workspace), special values included."""
    b, m, n = 8192, 128, 4096
    X = cast_fp8(synth.normal(137, synth.T_X, (b, m)), us.E4M3)
    W = cast_fp8(synth.normal(137, synth.T_W1, (m, n)), us.E4M3)
    X[5, :] = 0x7E                      # 448 everywhere ...
    W[:, :2] = 0x7E                     # ... times 448 / -448 columns: +-inf in the FP16 Z
    W[:, 1] = 0xFE
    X[6, 3] = 0x7F                      # a NaN operand -> NaN in a whole row of Z
    X[7, :] = 0                         # zeros
    Z0, _, H0 = linear_fwd(X, W, us.E4M3, us.E4M3, epi=us.EPI_GELU, want16=False, want8=True)
    Z1, _, H1 = linear_fwd(X, W, us.E4M3, us.E4M3, epi=us.EPI_GELU, want16=False, want8=True,
                           workspace_bytes=us.workspace_bytes(b, m, n))
    assert np.array_equal(Z0.view(np.uint16), Z1.view(np.uint16))
    assert np.isinf(Z0[5].astype(np.float32)).any() and np.isnan(Z0[6].astype(np.float32)).all()
    assert np.array_equal(H0, H1)
    # sampled rows against the oracle as well (the codes may differ by one where FP32 GELU flipped an FP16 tie)
    rows = [0, 1, 7, 100, 4095, 8191]
    ref = O.cast_fp8(O.gelu_fwd(Z1[rows], O.gelu_scales()[0]), O.E4M3)[0]
    d = np.abs(H1[rows].astype(np.int32) - ref.astype(np.int32))
    assert d.max() <= 1 and np.mean(d != 0) < 1e-3

    # grad_X with GELU': output [b, m] must be large, the reduction n short
    b, m, n = 8192, 4096, 128
    G = cast_fp8(synth.normal(139, synth.T_G, (b, n)), us.E5M2)
    W = cast_fp8(synth.normal(139, synth.T_W1, (m, n)), us.E4M3)
    Zpre = synth.normal(139, 7, (b, m), sigma=2.0)
    special = np.array([np.nan, np.inf, -np.inf, 0.0, -0.0, 6e-8, -6e-8, 8.0, -8.0, 8.01, -8.01, 65504.0, -65504.0, 7.996],
                       np.float16)
    Zpre[3, :special.size] = special
    args = dict(epi=us.EPI_GELU_GRAD, Zpre=Zpre, want8=True, do_dw=False)
    dZ0, _, c0 = linear_bwd(None, W, G, us.E4M3, us.E4M3, us.E5M2, no_workspace=True, **args)
    dZ1, _, c1 = linear_bwd(None, W, G, us.E4M3, us.E4M3, us.E5M2, **args)
    same = (dZ0.view(np.uint16) == dZ1.view(np.uint16)) | (np.isnan(dZ0.astype(np.float32)) & np.isnan(dZ1.astype(np.float32)))
    assert same.all()
    assert np.isnan(dZ1[3, :3].astype(np.float32)).all() and np.isfinite(dZ1[3, 3:special.size].astype(np.float32)).all()
    ok = ~np.isnan(dZ0.astype(np.float32))
    assert np.array_equal(c0[ok], c1[ok])
    rows = [0, 3, 4, 4095, 8191]
    dH = O.linear_bwd_dx(G[rows], W, n ** -0.5, O.E5M2, O.E4M3)
    ref = O.gelu_bwd(Zpre[rows], dH, O.gelu_scales()[1])
    fin = np.isfinite(ref.astype(np.float32))
    assert_close(np.where(fin, dZ1[rows], 0), np.where(fin, ref, 0), "dZ (table)", fp8=True)


def test_table_driven_gelu_fp16_output_equals_the_arithmetic_one():
    """FP16 operands, FP16 activation out: the table (|z| <= 6, both signs) plus its closed forms beyond
    must reproduce the arithmetic epilogue bit for bit.  Z is steered through every interesting value by
    a one-hot X row block: Z[i, j] = W[k(i), j] exactly (alpha = 1)."""
    b, m, n = 8192, 64, 4096                         # 32 x 16 tiles of 256: the table path
    vals = np.arange(65536, dtype=np.uint32).astype(np.uint16).view(np.float16)      # every FP16 pattern
    W = vals.reshape(16, 4096).copy()                # 16 reduction rows hold all 65536 patterns
    W[~np.isfinite(W.astype(np.float32))] = 0        # (0 * inf would poison whole columns; see below)
    W = np.concatenate([W, np.zeros((m - 16, n), np.float16)])
    W[16, :] = 65504.0
    X = np.zeros((b, m), np.float16)
    X[np.arange(b), np.arange(b) % 16] = 1.0         # row i selects reduction row i % 16
    X[4000, 16], X[4001, 16], X[4002, 3] = 2.0, -2.0, np.nan     # rows of +inf, -inf and NaN in Z
    kw = dict(alpha=1.0, epi=us.EPI_GELU, want16=True, want8=False)
    Z0, H0, _ = linear_fwd(X, W, us.F16, us.F16, **kw)
    Z1, H1, _ = linear_fwd(X, W, us.F16, us.F16, workspace_bytes=us.workspace_bytes(b, m, n), **kw)
    fin = np.ones((16, n), bool)
    assert np.array_equal(Z1[:16], W[:16]) and np.array_equal(Z0.view(np.uint16), Z1.view(np.uint16))   # Z is W (-0 -> +0)
    assert np.all(Z1[4000] == np.inf) and np.all(Z1[4001] == -np.inf) and np.isnan(Z1[4002].astype(np.float32)).all()
    assert np.all(H1[4000] == np.inf) and np.isnan(H1[4001].astype(np.float32)).all()
    nan0, nan1 = np.isnan(H0.astype(np.float32)), np.isnan(H1.astype(np.float32))
    assert np.array_equal(nan0, nan1)
    assert np.array_equal(H0.view(np.uint16)[~nan0], H1.view(np.uint16)[~nan1])
    # a quarter of everything: tiny negative products round to -0, which a sum of products cannot give
    kw["alpha"] = 0.25
    Zq0, Hq0, _ = linear_fwd(X, W, us.F16, us.F16, **kw)
    Zq1, Hq1, _ = linear_fwd(X, W, us.F16, us.F16, workspace_bytes=us.workspace_bytes(b, m, n), **kw)
    assert (Zq1[:16].view(np.uint16) == 0x8000).any()
    nq = np.isnan(Hq0.astype(np.float32))
    assert np.array_equal(nq, np.isnan(Hq1.astype(np.float32))) and np.array_equal(Hq0.view(np.uint16)[~nq], Hq1.view(np.uint16)[~nq])
    # and against the oracle on the 65536 distinct inputs (at most one FP16 ulp apart, rarely)
    ref = O.gelu_fwd(Z1[:16], O.gelu_scales()[0])
    ok = np.isfinite(ref.astype(np.float32)) & fin
    assert_close(np.where(ok, H1[:16], 0), np.where(ok, ref, 0), "H (table, FP16)")


@pytest.mark.parametrize("fp8", [False, True])
@pytest.mark.parametrize("shape", [(8192, 4096, 1024), (8192, 1024, 4096)])
def test_paired_grad_x_grad_w_launch_equals_separate_launches(fp8, shape):
    """A grad_X of large (or 256 x 128) tiles together with a grad_W of about one small tile per CU goes
    out as one launch.  Shapes: grad_X 8192 x 4096 (512 large tiles: the same kernel as alone, so the same
    bits) with grad_W 4096 x 1024, and grad_X 8192 x 1024 with grad_W 1024 x 4096.  In the pair grad_W sits
    on 128 tiles of 256 x 128 (alone: 256 of 128 x 128) and the second grad_X on the large tile; their wave
    groups share the k-steps differently, so the sums are added in another order: equal within the matmul
    tolerance, the same bits from call to call and whatever the epilogue of grad_X."""
    b, m, n = shape
    (X, W, G), gdt, odt = _operands(b, m, n, 149, fp8)
    Zpre = synth.normal(149, 7, (b, m))
    dW_first = None
    for epi in (us.EPI_NONE, us.EPI_GELU_GRAD):
        kw = dict(epi=epi, Zpre=Zpre if epi else None, want8=bool(epi) and fp8)
        dX, dW, c8 = linear_bwd(X, W, G, *gdt, **kw)                       # paired
        dW_first = dW if dW_first is None else dW_first
        assert np.array_equal(dW.view(np.uint16), dW_first.view(np.uint16)), epi
        dX1, _, c81 = linear_bwd(None, W, G, *gdt, do_dw=False, **kw)
        _, dW1, _ = linear_bwd(X, None, G, *gdt, do_dx=False)
        if m >= 4096:
            assert np.array_equal(dX.view(np.uint16), dX1.view(np.uint16)), epi
            if c8 is not None:
                assert np.array_equal(c8, c81)
        else:      # the paired grad_X adds its k-steps in two interleaved halves: same sum, another order
            assert_close(dX, dX1, "dX paired vs separate", fp8=fp8)
            assert np.mean(dX.view(np.uint16) != dX1.view(np.uint16)) < 0.2
            if c8 is not None:     # the codes are those of this launch's own FP16 result
                assert np.array_equal(c8, O.cast_fp8(dX, O.E5M2)[0])
        assert_close(dW, dW1, "dW paired vs separate", fp8=fp8)
        assert np.mean(dW.view(np.uint16) != dW1.view(np.uint16)) < 0.2
    rows, cols = [0, 1, 4097, 8191], [0, 5, 1023]
    assert_close(dW[:, cols], O.linear_bwd_dw(X, np.ascontiguousarray(G[:, cols]), b ** -0.5, odt[0], odt[2]), "dW paired", fp8=fp8)
    dH = O.linear_bwd_dx(G[rows], W, n ** -0.5, odt[2], odt[1])
    assert_close(dX[rows], O.gelu_bwd(Zpre[rows], dH, O.gelu_scales()[1]), "dZ paired", fp8=fp8)
