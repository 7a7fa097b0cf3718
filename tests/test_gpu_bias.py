"""GPU parity for the bias row of the forward product (us_linear_bias_fwd, fused into every forward epilogue), its
gradient (us_bias_grad) and the FFN with biases (us_ffn_bias_fwd / us_ffn_bias_bwd), against the oracle."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2303_11257_amd as us
import synth
from gpu_util import DEV, assert_close, empty, ptr, stream, to_dev, to_np

pytestmark = pytest.mark.gpu


def _bits(a):
    return np.ascontiguousarray(a).view(np.uint16)


def _operands(b, m, n, seed, fp8):
    X, W, _ = synth.linear_inputs(b, m, n, seed)
    if fp8:
        return O.cast_fp8(X, O.E4M3)[0], O.cast_fp8(W, O.E4M3)[0], us.E4M3
    return X, W, us.F16


def _fwd(X, W, dt, bias, alpha=0.0, epi=us.EPI_NONE, epi_scale=0.0, skip=None, want16=False, want8=False, workspace=False):
    b, m = X.shape
    n = W.shape[1]
    tX, tW, tb = to_dev(X), to_dev(W), (to_dev(bias) if bias is not None else None)
    Y = empty((b, n), np.float16)
    a16 = to_dev(skip) if skip is not None else (empty((b, n), np.float16) if want16 else None)
    a8 = empty((b, n), np.uint8) if want8 else None
    wsb = us.TABLE_AREA_BYTES if workspace else 0
    ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device=DEV)
    us.linear_bias_fwd(ptr(tX), ptr(tW), ptr(tb), ptr(Y), b, m, n, dt, dt, us.F16, alpha, epi, epi_scale, ptr(a16), ptr(a8),
                       ptr(ws) if workspace else None, wsb, stream())
    return to_np(Y), (to_np(a16) if want16 else None), (to_np(a8) if want8 else None)


# staged kernel (ragged K), 128 x 128 direct tiles with a ragged edge, the wave-split tile (few tiles, long K), 256 x 256 tiles
SHAPES = [(48, 80, 112), (272, 256, 400), (1024, 1024, 2048), (4096, 128, 6144)]


@pytest.mark.parametrize("fp8", [False, True])
@pytest.mark.parametrize("shape", SHAPES)
def test_linear_bias_fwd_against_the_oracle(shape, fp8):
    b, m, n = shape
    X, W, dt = _operands(b, m, n, 71, fp8)
    bias = synth.normal(71, 9, (n,), sigma=0.75)
    Y, _, _ = _fwd(X, W, dt, bias)
    odt = O.E4M3 if fp8 else O.F16
    ref = O.linear_fwd(X, W, O.linear_scales(b, m, n)[0], odt, odt, bias=bias)
    assert_close(Y, ref, f"Y {shape}", fp8=fp8)
    # without the bias the call is us_linear_fwd bit for bit, and a zero bias changes nothing either
    Y0, _, _ = _fwd(X, W, dt, None)
    Yz, _, _ = _fwd(X, W, dt, np.zeros(n, np.float16))
    tX, tW, Yp = to_dev(X), to_dev(W), empty((b, n), np.float16)
    us.linear_fwd(ptr(tX), ptr(tW), ptr(Yp), b, m, n, dt, dt, us.F16, 0.0, us.EPI_NONE, 0.0, None, None, None, 0, stream())
    assert np.array_equal(_bits(Y0), _bits(to_np(Yp))) and np.array_equal(_bits(Yz), _bits(Y0))
    assert not np.array_equal(_bits(Y), _bits(Y0))


@pytest.mark.parametrize("shape", [(64, 64, 96), (272, 256, 400), (512, 1024, 1024)])
def test_exact_integers_with_bias(shape):
    b, m, n = shape
    X = synth.small_ints(72, synth.T_X, (b, m))
    W = synth.small_ints(72, synth.T_W1, (m, n))
    bias = synth.small_ints(72, 9, (n,), lo=-8, hi=8)
    Y, _, _ = _fwd(X, W, us.F16, bias, alpha=0.25)
    ref = O.linear_fwd(X, W, 0.25, bias=bias)
    assert np.array_equal(_bits(Y), _bits(ref))
    exact = (0.25 * (X.astype(np.float64) @ W.astype(np.float64)) + bias.astype(np.float64)).astype(np.float16)
    assert np.array_equal(_bits(Y), _bits(exact))


def test_bias_is_added_before_the_single_rounding():
    # alpha * XW = 1 + 2^-11 in every element: alone it rounds to 1; the bias 2^-12 tips the unrounded sum up
    b, m, n = 32, 16, 32
    X = np.zeros((b, m), np.float16); X[:, 0] = 1.0; X[:, 1] = 1.0
    W = np.zeros((m, n), np.float16); W[0, :] = 1.0; W[1, :] = 2.0 ** -11
    bias = np.full(n, 2.0 ** -12, np.float16)
    Y, _, _ = _fwd(X, W, us.F16, bias, alpha=1.0)
    assert np.all(Y.astype(np.float64) == 1.0 + 2.0 ** -10)
    Y0, _, _ = _fwd(X, W, us.F16, None, alpha=1.0)
    assert np.all(Y0 == 1.0)


@pytest.mark.parametrize("fp8", [False, True])
def test_gelu_and_residual_epilogues_act_on_the_biased_output(fp8):
    b, m, n = 272, 256, 400
    X, W, dt = _operands(b, m, n, 73, fp8)
    odt = O.E4M3 if fp8 else O.F16
    bias = synth.normal(73, 9, (n,), sigma=0.75)
    Z, H16, H8 = _fwd(X, W, dt, bias, epi=us.EPI_GELU, want16=True, want8=fp8)
    assert_close(Z, O.linear_fwd(X, W, O.linear_scales(b, m, n)[0], odt, odt, bias=bias), "Z", fp8=fp8)
    Href = O.gelu_fwd(Z, O.gelu_scales()[0])
    assert np.max(np.abs(_bits(H16).astype(np.int64) - _bits(Href).astype(np.int64))) <= 1
    if fp8:
        assert np.array_equal(H8, O.cast_fp8(H16, O.E4M3)[0])
    skip = synth.normal(73, 10, (b, n))
    tau = 0.3
    Out, _, _ = _fwd(X, W, dt, bias, epi=us.EPI_RESIDUAL, epi_scale=float(np.sqrt(tau)), skip=skip)
    Yb, _, _ = _fwd(X, W, dt, bias)              # the intermediate the fused epilogue rounds to FP16: same kernel, same bits
    sw, bw = O.residual_weights(tau)
    assert_close(Out, O.weighted_add2(skip, Yb, sw, bw), "Out")


def test_table_driven_gelu_with_bias_matches_the_arithmetic_epilogue():
    b, m, n = 4096, 128, 6144                    # 384 tiles of 256 x 256: the large tile, so the table path is taken
    X, W, dt = _operands(b, m, n, 74, True)
    bias = synth.normal(74, 9, (n,), sigma=0.75)
    Zt, _, Ht = _fwd(X, W, dt, bias, epi=us.EPI_GELU, want8=True, workspace=True)
    Za, _, Ha = _fwd(X, W, dt, bias, epi=us.EPI_GELU, want8=True, workspace=False)
    assert np.array_equal(_bits(Zt), _bits(Za)) and np.array_equal(Ht, Ha)
    rows = np.arange(0, b, 97)
    ref = O.linear_fwd(X[rows], W, O.linear_scales(b, m, n)[0], O.E4M3, O.E4M3, bias=bias)
    assert_close(Zt[rows], ref, "Z (table path)", fp8=True)


def _sum_close(gpu, ref):
    """Column sums: FP32 on the GPU (blocks of 32 rows, then the blocks), double in the oracle.  The difference is one
    FP16 step of the result where a rounding flips, plus, where a sum cancels to nearly nothing, the absolute error of
    the FP32 additions (~1e-6 after the b^-1/2 factor), which is then many steps of a tiny result."""
    g, r = gpu.astype(np.float64), ref.astype(np.float64)
    return bool(np.all(np.abs(g - r) <= 2.0 ** -10 * np.abs(r) + 2e-5))


def _bias_grad(G, g_dt, beta=0.0):
    b, n = G.shape
    tG = to_dev(G)
    dc = empty((n,), np.float16)
    wsb = us.bias_grad_workspace_bytes(b, n)
    ws = torch.full((max(wsb, 16),), 0xA5, dtype=torch.uint8, device=DEV)
    us.bias_grad(ptr(tG), g_dt, ptr(dc), b, n, beta, ptr(ws), wsb, stream())
    return to_np(dc)


@pytest.mark.parametrize("fmt", ["f16", "e5m2", "e4m3"])
@pytest.mark.parametrize("shape", [(1, 16), (37, 48), (1000, 768), (4096, 4096), (8192, 1024), (77, 8192), (70001, 32), (140000, 16)])
def test_bias_grad_against_the_oracle(shape, fmt):
    b, n = shape
    G = synth.normal(75, synth.T_G, (b, n))
    if fmt == "f16":
        Gop, gdt, odt = G, us.F16, O.F16
    elif fmt == "e5m2":
        Gop, gdt, odt = O.cast_fp8(G, O.E5M2)[0], us.E5M2, O.E5M2
    else:
        Gop, gdt, odt = O.cast_fp8(G, O.E4M3)[0], us.E4M3, O.E4M3
    dc = _bias_grad(Gop, gdt)
    ref = O.bias_grad(Gop, O.bias_scale(b), g_dt=odt)
    assert _sum_close(dc, ref)
    assert np.mean(_bits(dc) != _bits(ref)) < 0.01
    assert np.array_equal(_bits(dc), _bits(_bias_grad(Gop, gdt)))                            # fixed order of additions


def test_bias_grad_of_no_rows_is_zero():
    dc = torch.full((48,), 7.0, dtype=torch.float16, device=DEV)
    us.bias_grad(None, us.F16, ptr(dc), 0, 48, 0.0, None, 0, stream())
    assert not to_np(dc).any()


def test_bias_grad_exact_integers():
    b, n = 1000, 304
    G = synth.small_ints(76, synth.T_G, (b, n))
    dc = _bias_grad(G, us.F16, beta=2.0 ** -4)
    exact = (G.astype(np.float64).sum(axis=0) / 16).astype(np.float16)
    assert np.array_equal(_bits(dc), _bits(exact)) and np.array_equal(_bits(dc), _bits(O.bias_grad(G, 2.0 ** -4)))


def _ffn_bias_run(T, d, f, seed, fp8, tables=False, store_dz16=True):
    X, W1, W2, G = synth.ffn_inputs(T, d, f, seed)
    b1, b2 = synth.normal(seed, 11, (f,), sigma=0.5), synth.normal(seed, 12, (d,), sigma=0.5)
    dev = {k: to_dev(v) for k, v in dict(X=X, W1=W1, W2=W2, G=G, b1=b1, b2=b2).items()}
    st = stream()
    for k, fmt in (("X", us.E4M3), ("W1", us.E4M3), ("W2", us.E4M3), ("G", us.E5M2)):
        if fp8:
            dst = torch.empty(dev[k].shape, dtype=torch.uint8, device=DEV)
            us.cast_fp8(ptr(dev[k]), us.F16, ptr(dst), fmt, dev[k].numel(), 1.0, None, st)
            dev[k + "op"] = dst
        else:
            dev[k + "op"] = dev[k]
    e = lambda shape, dt=torch.float16: torch.empty(shape, dtype=dt, device=DEV)
    dev["Z"], dev["Y"], dev["H"] = e((T, f)), e((T, d)), e((T, f), torch.uint8 if fp8 else torch.float16)
    dev["dZ16"], dev["dX"], dev["dW1"], dev["dW2"], dev["db1"], dev["db2"] = e((T, f)), e((T, d)), e((d, f)), e((f, d)), e((f,)), e((d,))
    dev["dZ8"] = e((T, f), torch.uint8) if fp8 else None
    wsb = us.ffn_bias_workspace_bytes(T, d, f)
    ws = torch.full((wsb,), 0xA5, dtype=torch.uint8, device=DEV)
    mode = us.FFN_FP8 if fp8 else 0
    if tables:
        us.gelu_tables(ptr(ws), wsb, 0.0, 0.0, st)
        mode |= us.FFN_TABLES_READY
    us.ffn_bias_fwd(ptr(dev["Xop"]), ptr(dev["W1op"]), ptr(dev["b1"]), ptr(dev["W2op"]), ptr(dev["b2"]), ptr(dev["Z"]), ptr(dev["H"]),
                    ptr(dev["Y"]), T, d, f, mode, ptr(ws), wsb, st)
    us.ffn_bias_bwd(ptr(dev["Xop"]), ptr(dev["W1op"]), ptr(dev["W2op"]), ptr(dev["Z"]), ptr(dev["H"]), ptr(dev["Gop"]), ptr(dev["G"]),
                    ptr(dev["dZ16"]) if store_dz16 else None, ptr(dev["dZ8"]), ptr(dev["dX"]), ptr(dev["dW1"]), ptr(dev["dW2"]), ptr(dev["db1"]),
                    ptr(dev["db2"]), T, d, f, mode, ptr(ws), wsb, st)
    torch.cuda.synchronize()
    return dev, dict(X=X, W1=W1, W2=W2, G=G, b1=b1, b2=b2)


@pytest.mark.parametrize("fp8", [False, True])
def test_ffn_with_biases_small_ragged_shape(fp8):
    T, d, f = 272, 144, 400
    dev, host = _ffn_bias_run(T, d, f, 77, fp8)
    g = {k: v.cpu().numpy() for k, v in dev.items() if v is not None}
    op, gr = (O.E4M3, O.E5M2) if fp8 else (O.F16, O.F16)
    a1, bx1, bw1 = O.linear_scales(T, d, f)
    a2, bx2, bw2 = O.linear_scales(T, f, d)
    ag, bg = O.gelu_scales()
    assert_close(g["Z"], O.linear_fwd(g["Xop"], g["W1op"], a1, op, op, bias=host["b1"]), "Z", fp8=fp8)
    Href = O.gelu_fwd(g["Z"], ag)
    if fp8:    # only the codes are stored: one code off where the FP32 GELU moved the FP16 value across an FP8 boundary
        diff = np.abs(g["H"].astype(np.int32) - O.cast_fp8(Href, O.E4M3)[0].astype(np.int32))
        assert diff.max() <= 1 and np.mean(diff != 0) < 1e-3
    else:
        assert_close(g["H"], Href, "H")
    assert_close(g["Y"], O.linear_fwd(g["H"], g["W2op"], a2, op, op, bias=host["b2"]), "Y", fp8=fp8)
    dH = O.linear_bwd_dx(g["Gop"], g["W2op"], bx2, gr, op)
    assert_close(g["dZ16"], O.gelu_bwd(g["Z"], dH, bg), "dZ", fp8=fp8)
    assert _sum_close(g["db2"], O.bias_grad(host["G"], O.bias_scale(T)))
    assert _sum_close(g["db1"], O.bias_grad(g["dZ16"], O.bias_scale(T)))
    dZop = g["dZ8"] if fp8 else g["dZ16"]
    assert_close(g["dX"], O.linear_bwd_dx(dZop, g["W1op"], bx1, gr, op), "dX", fp8=fp8)
    assert_close(g["dW1"], O.linear_bwd_dw(g["Xop"], dZop, bw1, op, gr), "dW1", fp8=fp8)
    assert_close(g["dW2"], O.linear_bwd_dw(g["H"], g["Gop"], bw2, op, gr), "dW2", fp8=fp8)


@pytest.mark.parametrize("shape,tables", [((272, 144, 400), False), ((1024, 256, 2048), True), ((4096, 1024, 3072), True),
                                          ((8192, 1024, 4096), True)])
def test_db1_needs_no_stored_fp16_dz(shape, tables):
    """The column sums of dZ are taken inside the epilogue that produces it: an FP8 step that stores only the E5M2 copy
    of dZ gives the same db1, bit for bit, and the same other outputs.  Shapes: staged kernel with ragged tiles,
    128 x 128 tiles, 256 x 128 tiles with two wave groups in a paired launch (arithmetic epilogue), the large tile with
    the table-driven epilogue in a paired launch."""
    T, d, f = shape
    a, _ = _ffn_bias_run(T, d, f, 79, True, tables=tables)
    b, _ = _ffn_bias_run(T, d, f, 79, True, tables=tables, store_dz16=False)
    for k in ("db1", "db2", "dZ8", "dX", "dW1", "dW2"):
        assert torch.equal(a[k].view(torch.uint8), b[k].view(torch.uint8)), k
    assert _sum_close(b["db1"].cpu().numpy(), O.bias_grad(a["dZ16"].cpu().numpy(), O.bias_scale(T)))


def test_ffn_with_biases_at_the_bert_large_shape_sampled():
    T, d, f = 8192, 1024, 4096
    dev, host = _ffn_bias_run(T, d, f, 20230313, True, tables=True)
    rows = np.array([0, 1, 255, 256, 4097, 8191])
    ridx = torch.as_tensor(rows, device=DEV)
    W1op, W2op = dev["W1op"].cpu().numpy(), dev["W2op"].cpu().numpy()
    a1, a2 = O.linear_scales(T, d, f)[0], O.linear_scales(T, f, d)[0]
    Zr = dev["Z"][ridx].cpu().numpy()
    assert_close(Zr, O.linear_fwd(dev["Xop"][ridx].cpu().numpy(), W1op, a1, O.E4M3, O.E4M3, bias=host["b1"]), "Z rows", fp8=True)
    assert_close(dev["Y"][ridx].cpu().numpy(), O.linear_fwd(dev["H"][ridx].cpu().numpy(), W2op, a2, O.E4M3, O.E4M3, bias=host["b2"]), "Y rows", fp8=True)
    assert _sum_close(dev["db2"].cpu().numpy(), O.bias_grad(host["G"], O.bias_scale(T)))
    assert _sum_close(dev["db1"].cpu().numpy(), O.bias_grad(dev["dZ16"].cpu().numpy(), O.bias_scale(T)))
    # unit variance of the bias gradients (b^-1/2 on a sum of T unit-scale rows); dZ has variance ~1 only where gelu' does
    assert abs(float(dev["db2"].float().std()) - 1.0) < 0.05
    assert 0.8 < float(dev["db1"].float().std()) < 1.2


def test_bias_and_its_gradient_propagate_nan():
    b, m, n = 64, 64, 96
    X, W, dt = _operands(b, m, n, 78, False)
    bias = synth.normal(78, 9, (n,))
    bias[5] = np.nan
    bias[7] = np.inf
    Y, _, _ = _fwd(X, W, dt, bias)
    assert np.all(np.isnan(Y[:, 5])) and np.all(np.isposinf(Y[:, 7])) and np.isfinite(np.delete(Y, [5, 7], axis=1)).all()
    G = synth.normal(78, synth.T_G, (b, n))
    G[3, 11] = np.nan
    dc = _bias_grad(G, us.F16)
    assert np.isnan(dc[11]) and np.isfinite(np.delete(dc, 11)).all()
