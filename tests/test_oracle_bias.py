"""Pins for the oracle's bias row (App. J.1: ffn(z) = W2 act(W1 z + b1) + b2) and its gradient (CPU only): exact
rational brute force, a zero matmul that must return the bias itself, index-coded rows that expose a bias applied
along the wrong axis, torch's float64 autograd for the whole biased FFN, and the unit variance of the gradient."""
from fractions import Fraction

import numpy as np
import torch

import oracle
import synth
from oracle import E4M3, E5M2, F16, F32


def _bits(a):
    return np.ascontiguousarray(a).view(np.uint16)


def _round_f16(fr: Fraction) -> int:
    v = fr.numerator / fr.denominator
    assert Fraction(v) == fr
    return int(np.array([v], np.float64).astype(np.float16).view(np.uint16)[0])


def test_tiny_shape_against_exact_rational_arithmetic():
    b, m, n = 5, 7, 3
    X = synth.normal(61, synth.T_X, (b, m))
    W = synth.normal(61, synth.T_W1, (m, n))
    c = synth.normal(61, synth.T_G, (n,))
    Y = oracle.linear_fwd(X, W, 0.375, bias=c)
    for i in range(b):
        for j in range(n):
            s = sum(Fraction(float(X[i, k])) * Fraction(float(W[k, j])) for k in range(m))
            assert _bits(Y)[i, j] == _round_f16(Fraction(3, 8) * s + Fraction(float(c[j]))), (i, j)
    G = synth.normal(61, synth.T_G, (b, n))
    dc = oracle.bias_grad(G, 0.5)
    for j in range(n):
        assert _bits(dc)[j] == _round_f16(Fraction(1, 2) * sum(Fraction(float(G[i, j])) for i in range(b)))


def test_zero_product_returns_the_bias_and_no_bias_is_the_plain_product():
    b, m, n = 6, 16, 48
    W = synth.normal(62, synth.T_W1, (m, n))
    c = synth.normal(62, synth.T_G, (n,), sigma=3.0)
    Y = oracle.linear_fwd(np.zeros((b, m), np.float16), W, 0.25, bias=c)
    assert np.array_equal(_bits(Y), np.broadcast_to(_bits(c), (b, n)))
    X = synth.normal(62, synth.T_X, (b, m))
    assert np.array_equal(_bits(oracle.linear_fwd(X, W, 0.25, bias=np.zeros(n, np.float16))), _bits(oracle.linear_fwd(X, W, 0.25)))
    # one rounding of the sum, not round(round(alpha * XW) + c): XW = 1 + 2^-11 is a tie that rounds to 1 on its
    # own, and the bias 2^-12 then changes nothing; added before the rounding it tips the sum up to 1 + 2^-10
    X1 = np.array([[1.0, 1.0]], np.float16)
    W1 = np.array([[1.0], [2.0 ** -11]], np.float16)
    c1 = np.array([2.0 ** -12], np.float16)
    assert float(oracle.linear_fwd(X1, W1, 1.0)[0, 0]) == 1.0
    assert float(oracle.linear_fwd(X1, W1, 1.0, bias=c1)[0, 0]) == 1.0 + 2.0 ** -10


def test_bias_runs_along_the_output_features_not_the_rows():
    b, m, n = 4, 16, 12
    X = np.zeros((b, m), np.float16)
    W = np.zeros((m, n), np.float16)
    c = np.arange(1, n + 1).astype(np.float16)
    Y = oracle.linear_fwd(X, W, 1.0, bias=c)
    assert Y.shape == (b, n) and all(np.array_equal(Y[i], c) for i in range(b))
    G = (np.arange(b)[:, None] * 100 + np.arange(n)[None, :]).astype(np.float16)     # G[i,j] = 100 i + j
    dc = oracle.bias_grad(G, 1.0, out_dt=F32)
    assert dc.shape == (n,) and np.array_equal(dc, 100.0 * (b * (b - 1) // 2) + b * np.arange(n))


def test_fp8_inputs_decode_before_the_sum():
    b, n = 64, 32
    G = synth.normal(63, synth.T_G, (b, n))
    G8, _ = oracle.cast_fp8(G, E5M2)
    dc = oracle.bias_grad(G8, 0.125, g_dt=E5M2, out_dt=F32)
    ref = (0.125 * oracle.decode(G8, E5M2).sum(axis=0)).astype(np.float32)
    assert np.array_equal(dc, ref)


def test_whole_biased_ffn_against_float64_autograd():
    """FP16 storage, so the oracle's stage-wise roundings bound the difference: every tensor within a few FP16 steps of
    the float64 chain differentiated by torch."""
    T, d, f = 96, 32, 64
    X, W1, W2, G = synth.ffn_inputs(T, d, f, 64)
    b1 = synth.normal(64, 11, (f,), sigma=0.5)
    b2 = synth.normal(64, 12, (d,), sigma=0.5)
    fw = oracle.ffn_fwd(X, W1, W2, False, b1=b1, b2=b2)
    bw = oracle.ffn_bwd(X, W1, W2, G, fw, False, with_bias=True)
    ag, bg = (float(v) for v in oracle.gelu_scales())
    t = lambda a: torch.tensor(a.astype(np.float64), requires_grad=True)
    x, w1, w2, c1, c2 = t(X), t(W1), t(W2), t(b1), t(b2)
    z = x @ w1 * d ** -0.5 + c1
    h = ag * z * 0.5 * (1 + torch.erf(z / 2 ** 0.5))
    y = h @ w2 * f ** -0.5 + c2
    assert np.abs(fw["Z"].astype(np.float64) - z.detach().numpy()).max() < 2e-3 * 4
    assert np.abs(fw["Y"].astype(np.float64) - y.detach().numpy()).max() < 4e-3 * 4
    # the unit-scaled backward pass is not the plain chain rule (each op has its own backward factor), so compare
    # the bias gradients with autograd of the matching unscaled pieces: d(sum(G*y))/dc2 = column sums of G
    (y * torch.tensor(G.astype(np.float64))).sum().backward()
    assert np.allclose(bw["db2"].astype(np.float64), T ** -0.5 * c2.grad.numpy(), rtol=2e-3, atol=1e-3)
    # db1 = beta * column sums of dZ, and dZ is the oracle's own (scaled) gradient at Z
    assert np.allclose(bw["db1"].astype(np.float64), T ** -0.5 * bw["dZ"].astype(np.float64).sum(axis=0), rtol=2e-3, atol=1e-3)
    # autograd: dL/dz = (G w2^T f^-1/2) * alpha_g gelu'(z); unit-scaled backward: (G w2^T d^-1/2) * beta_g gelu'(z)
    # (grad_X of layer 2 has fan-out d).  With that ratio undone autograd's dc1 is the same column sum.
    auto = c1.grad.numpy() * (bg / ag) * (d ** -0.5 / f ** -0.5) * T ** -0.5
    assert np.allclose(bw["db1"].astype(np.float64), auto, rtol=2e-2, atol=2e-2)


def test_bias_gradient_has_unit_variance_for_unit_gradients():
    b, n = 4096, 2048
    G = synth.normal(65, synth.T_G, (b, n))
    dc = oracle.bias_grad(G).astype(np.float64)
    assert oracle.bias_scale(b) == np.float32(b ** -0.5)
    assert abs(dc.std() - 1.0) < 0.05 and abs(dc.mean()) < 0.1
