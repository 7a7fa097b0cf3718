"""Pins for the oracle's scaled matmuls (CPU only): scale formulas as printed, exact rational
brute force on tiny shapes, index-coded operands that expose a transposed or mis-indexed operand,
numpy's float64 matmul as the textbook special case, and the unit-variance property at C1."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
import synth
from oracle import E4M3, E5M2, F16, F32


def test_scale_formulas_table_a2_and_sec_5_5():
    a, bx, bw = oracle.linear_scales(256, 256, 1024)           # the C1 shape
    assert (a, bx, bw) == (np.float32(1 / 16), np.float32(1 / 32), np.float32(1 / 16))
    b, m, n = 8192, 1024, 4096
    a, bx, bw = oracle.linear_scales(b, m, n)
    assert a == np.float32(m ** -0.5) and bx == np.float32(n ** -0.5) and bw == np.float32(b ** -0.5)
    a1, bx1, bw1 = oracle.linear_scales(b, m, n, mode=1)       # X is not a cut-edge: alpha = beta_1 = (mn)^-1/4
    assert a1 == bx1 == np.float32((m * n) ** -0.25) and bw1 == bw
    assert abs(float(a1) ** 2 - float(a) * float(bx)) < 1e-9  # geometric mean of the two
    a, bx, bw = oracle.linear_scales(100, 300, 700)
    assert np.allclose([a, bx, bw], [300 ** -0.5, 700 ** -0.5, 100 ** -0.5], rtol=1e-7)


def test_flop_overhead_formula_app_i2():
    """Rescaling cost relative to the three matmuls; the paper's 0.2 % for BERT-large."""
    b, m, n = 8192, 1024, 4096
    ratio = (b * m + m * n + b * n) / (6 * b * m * n)
    assert abs(ratio - (1 / b + 1 / m + 1 / n) / 6) < 1e-15
    assert ratio <= 1 / (2 * min(b, m, n))
    assert round(100 * 4 / (2 * 1024), 1) == 0.2


def _exact_round_f16(fr: Fraction) -> int:
    """RNE of an exact rational to FP16 bits, through numpy's double->half (the double is exact here)."""
    v = fr.numerator / fr.denominator
    assert Fraction(v) == fr
    return int(np.array([v], np.float64).astype(np.float16).view(np.uint16)[0])


def _frac(a):
    return [[Fraction(float(v)) for v in row] for row in a]


@pytest.mark.parametrize("fp8", [False, True])
def test_tiny_shapes_against_exact_rational_dot_products(fp8):
    b, m, n = 5, 7, 3
    X = synth.normal(41, synth.T_X, (b, m))
    W = synth.normal(41, synth.T_W1, (m, n))
    G = synth.normal(41, synth.T_G, (b, n))
    if fp8:
        X8, _ = oracle.cast_fp8(X, E4M3)
        W8, _ = oracle.cast_fp8(W, E4M3)
        G8, _ = oracle.cast_fp8(G, E5M2)
        Xv, Wv, Gv = oracle.decode(X8, E4M3), oracle.decode(W8, E4M3), oracle.decode(G8, E5M2)
        Y = oracle.linear_fwd(X8, W8, 0.5, E4M3, E4M3)
        dX = oracle.linear_bwd_dx(G8, W8, 0.25, E5M2, E4M3)
        dW = oracle.linear_bwd_dw(X8, G8, 2.0, E4M3, E5M2)
    else:
        Xv, Wv, Gv = X, W, G
        Y = oracle.linear_fwd(X, W, 0.5)
        dX = oracle.linear_bwd_dx(G, W, 0.25)
        dW = oracle.linear_bwd_dw(X, G, 2.0)
    Xf, Wf, Gf = _frac(Xv), _frac(Wv), _frac(Gv)
    for i in range(b):
        for j in range(n):
            s = sum(Xf[i][k] * Wf[k][j] for k in range(m))
            assert int(Y.view(np.uint16)[i, j]) == _exact_round_f16(Fraction(1, 2) * s)
        for k in range(m):
            s = sum(Gf[i][j] * Wf[k][j] for j in range(n))
            assert int(dX.view(np.uint16)[i, k]) == _exact_round_f16(Fraction(1, 4) * s)
    for k in range(m):
        for j in range(n):
            s = sum(Xf[i][k] * Gf[i][j] for i in range(b))
            assert int(dW.view(np.uint16)[k, j]) == _exact_round_f16(2 * s)


def test_index_coded_operands_expose_transposes():
    """X[i,k] = (i + 2k) mod 5 - 2 and one-hot / permutation weights: every product is an integer
    and each output names the operand element it came from."""
    b, m, n = 6, 8, 8
    i, k = np.meshgrid(np.arange(b), np.arange(m), indexing="ij")
    X = (((i + 2 * k) % 5) - 2).astype(np.float16)
    perm = np.array([3, 0, 7, 1, 6, 2, 5, 4])
    W = np.zeros((m, n), np.float16)
    W[np.arange(m), perm] = 1.0                                   # Y[:, perm[k]] = X[:, k]
    Y = oracle.linear_fwd(X, W, 1.0, out_dt=F32)
    assert np.array_equal(Y[:, perm], X.astype(np.float32))
    G = (((3 * i[:, :n] + k[:, :n]) % 5) - 2).astype(np.float16)  # G[b,n]
    dX = oracle.linear_bwd_dx(G, W, 1.0, out_dt=F32)              # dX[:, k] = G[:, perm[k]]
    assert np.array_equal(dX, G[:, perm].astype(np.float32))
    # rectangular, non-symmetric shapes so that a swapped dimension cannot pass
    b, m, n = 4, 3, 5
    X = np.arange(b * m).reshape(b, m).astype(np.float16) - 5
    G = (np.arange(b * n).reshape(b, n) % 7).astype(np.float16) - 3
    W = (np.arange(m * n).reshape(m, n) % 4).astype(np.float16) - 1
    Xd, Gd, Wd = X.astype(np.float64), G.astype(np.float64), W.astype(np.float64)
    assert np.array_equal(oracle.linear_fwd(X, W, 1.0, out_dt=F32), (Xd @ Wd).astype(np.float32))
    assert np.array_equal(oracle.linear_bwd_dx(G, W, 1.0, out_dt=F32), (Gd @ Wd.T).astype(np.float32))
    assert np.array_equal(oracle.linear_bwd_dw(X, G, 1.0, out_dt=F32), (Xd.T @ Gd).astype(np.float32))


def test_unit_alpha_fp32_output_is_the_textbook_matmul():
    b, m, n = 37, 129, 53
    X, W, G = synth.linear_inputs(b, m, n, seed=43)
    Xd, Wd, Gd = (a.astype(np.float64) for a in (X, W, G))
    for got, want in ((oracle.linear_fwd(X, W, 1.0, out_dt=F32), Xd @ Wd),
                      (oracle.linear_bwd_dx(G, W, 1.0, out_dt=F32), Gd @ Wd.T),
                      (oracle.linear_bwd_dw(X, G, 1.0, out_dt=F32), Xd.T @ Gd)):
        assert got.shape == want.shape
        assert np.max(np.abs(got - want) / np.maximum(np.abs(want), 1.0)) < 2e-7   # one FP32 rounding


def test_scale_multiplies_before_the_single_rounding():
    """alpha*acc is rounded once: scaling by 2^-k commutes with FP16 rounding only while normal."""
    X, W, _ = synth.linear_inputs(16, 64, 32, seed=47)
    Y1 = oracle.linear_fwd(X, W, 1.0, out_dt=F32).astype(np.float64)
    Y = oracle.linear_fwd(X, W, 0.125)
    with np.errstate(over="ignore"):
        assert np.array_equal(Y.view(np.uint16), (0.125 * Y1).astype(np.float16).view(np.uint16))
    # FP16 output overflows to infinity (IEEE), it is not clamped
    big = np.full((2, 4), 300.0, np.float16)
    Yb = oracle.linear_fwd(big, big.T.copy(), 1.0)
    assert np.all(np.isinf(Yb.astype(np.float32)))


@pytest.mark.parametrize("fp8", [False, True])
def test_unit_variance_at_c1(fp8):
    """Var(XW) = m, Var(GW^T) = n, Var(X^T G) = b for unit-variance inputs (App. E.1), hence 1
    after the unconstrained scales; 5 % gate, standard error here is below 0.6 %."""
    b, m, n = 256, 256, 1024
    X, W, G = synth.linear_inputs(b, m, n, seed=synth.CONFIGS["C1"]["seed"])
    a, bx, bw = oracle.linear_scales(b, m, n)
    if fp8:
        X8, W8, G8 = oracle.cast_fp8(X, E4M3)[0], oracle.cast_fp8(W, E4M3)[0], oracle.cast_fp8(G, E5M2)[0]
        Y = oracle.linear_fwd(X8, W8, a, E4M3, E4M3)
        dX = oracle.linear_bwd_dx(G8, W8, bx, E5M2, E4M3)
        dW = oracle.linear_bwd_dw(X8, G8, bw, E4M3, E5M2)
    else:
        Y = oracle.linear_fwd(X, W, a)
        dX = oracle.linear_bwd_dx(G, W, bx)
        dW = oracle.linear_bwd_dw(X, G, bw)
    for t in (Y, dX, dW):
        v = float(np.var(t.astype(np.float64)))
        assert abs(v - 1.0) < 0.05, v
    # unscaled products carry the fan-in / fan-out / batch factor
    raw = oracle.linear_fwd(X, W, 1.0, out_dt=F32).astype(np.float64)
    assert abs(np.var(raw) / m - 1.0) < 0.05
    # the constrained (geometric-mean) scales do NOT give unit variance on this shape: 0.5 and 2
    a1, bx1, _ = oracle.linear_scales(b, m, n, mode=1)
    Yc = oracle.linear_fwd(X, W, a1).astype(np.float64)
    assert abs(np.var(Yc) - 0.5) < 0.05
