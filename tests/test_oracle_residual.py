"""Weighted addition and the residual FFN layer of the oracle (CPU only; Sec. 5.3, Table A.2, Fig. 3 right)."""
import math

import numpy as np
import pytest
from scipy.special import erf

import oracle
import synth


def test_weighted_add_scale_rule():
    """Table A.2: alpha = (sum gamma_i^2)^-1/2, beta_i = 1/gamma_i.  For the fixed(tau) weights the squares add up to
    one, so the interpolation needs no further output scale; a plain two-way add needs 2^-1/2."""
    for tau in (0.1, 0.25, 0.5, 0.9):
        a, betas = oracle.weighted_add_scales([math.sqrt(1 - tau), math.sqrt(tau)])
        assert abs(a - 1.0) < 1e-12
        assert abs(betas[0] - (1 - tau) ** -0.5) < 1e-12 and abs(betas[1] - tau ** -0.5) < 1e-12
    a, betas = oracle.weighted_add_scales([1.0, 1.0])
    assert abs(a - 2 ** -0.5) < 1e-15 and betas == [1.0, 1.0]
    a, _ = oracle.weighted_add_scales([3.0, 4.0])
    assert a == 0.2


def test_residual_weights_are_floats_whose_squares_sum_to_one():
    for tau in (0.0, 0.05, 0.36, 0.5, 1.0):
        skip, branch = oracle.residual_weights(tau)
        assert skip.dtype == np.float32 and branch.dtype == np.float32
        assert abs(float(skip) ** 2 + float(branch) ** 2 - 1.0) < 2e-7
        assert abs(float(branch) - math.sqrt(tau)) < 1e-7
    assert oracle.residual_weights(0.36)[1] == np.float32(0.6)


def test_weighted_add2_is_one_rounding_of_the_exact_sum():
    """Against numpy: the sum formed in float64 (exact for FP16 inputs and float weights: 11 + 24 bit products,
    two terms) and numpy's own round-to-nearest-even conversion to FP16."""
    a = synth.normal(71, 1, (64, 48))
    b = synth.normal(71, 2, (64, 48), sigma=3.0)
    for ca, cb in ((0.8, 0.6), (1.0, 0.0), (0.0, 1.0), (0.31622776, 0.94868330), (-1.0, 1.0)):
        want = (np.float64(np.float32(ca)) * a.astype(np.float64) + np.float64(np.float32(cb)) * b.astype(np.float64)).astype(np.float16)
        got = oracle.weighted_add2(a, b, ca, cb)
        assert np.array_equal(got.view(np.uint16), want.view(np.uint16)), (ca, cb)
    # identity and special values: weight 1 / 0 passes subnormals, the largest value and signed zero through
    s = np.array([6e-8, -6e-8, 65504.0, -65504.0, 0.0, -0.0, 1.0], np.float16)
    z = np.zeros_like(s)
    assert np.array_equal(oracle.weighted_add2(s, z, 1.0, 0.0).view(np.uint16)[:4], s.view(np.uint16)[:4])
    # overflow of the FP16 result is IEEE (inf), as for every FP16 output
    assert np.isinf(oracle.weighted_add2(np.array([65504.0], np.float16), np.array([65504.0], np.float16), 0.8, 0.6))[0]
    # FP32 storage as well
    a32, b32 = a.astype(np.float32), b.astype(np.float32)
    want = (np.float64(np.float32(0.8)) * a32.astype(np.float64) + np.float64(np.float32(0.6)) * b32.astype(np.float64)).astype(np.float32)
    assert np.array_equal(oracle.weighted_add2(a32, b32, 0.8, 0.6), want)


@pytest.mark.parametrize("tau", [0.1, 0.5, 0.8])
def test_interpolation_of_independent_unit_tensors_is_unit_variance(tau):
    a = synth.normal(73, 1, (512, 512))
    b = synth.normal(73, 2, (512, 512))
    skip, branch = oracle.residual_weights(tau)
    out = oracle.weighted_add2(a, b, skip, branch)
    assert abs(np.var(out.astype(np.float64)) - 1.0) < 0.02


def test_tau_zero_and_one_are_the_two_inputs():
    T, d, f = 32, 16, 48
    X, W1, W2, G = synth.ffn_inputs(T, d, f, seed=79)
    r0 = oracle.ffn_res_fwd(X, W1, W2, 0.0, False)
    assert np.array_equal(r0["Out"], X)
    r1 = oracle.ffn_res_fwd(X, W1, W2, 1.0, False)
    assert np.array_equal(r1["Out"], r1["Y"])
    b0 = oracle.ffn_res_bwd(X, W1, W2, G, r0, 0.0, False)
    assert np.array_equal(b0["dXin"], G)
    # the branch's own gradients do not depend on tau (its weight is moved out of its backward pass)
    b1 = oracle.ffn_res_bwd(X, W1, W2, G, r1, 1.0, False)
    for k in ("dW1", "dW2", "dZ", "dX"):
        assert np.array_equal(b0[k], b1[k]), k
    assert np.array_equal(b1["dXin"], b1["dX"])


def _f64_layer(X, W1, W2, tau, ag):
    """The residual layer as a plain float64 function: the textbook formulas, no rounding."""
    T, d = X.shape
    f = W1.shape[1]
    Z = X @ W1 / math.sqrt(d)
    H = ag * Z * 0.5 * (1.0 + erf(Z / math.sqrt(2.0)))
    Y = H @ W2 / math.sqrt(f)
    return math.sqrt(1 - tau) * X + math.sqrt(tau) * Y


def _fd_grad(fn, A, eps=1e-5):
    g = np.zeros_like(A)
    for idx in np.ndindex(*A.shape):
        old = A[idx]
        A[idx] = old + eps
        up = fn()
        A[idx] = old - eps
        dn = fn()
        A[idx] = old
        g[idx] = (up - dn) / (2 * eps)
    return g


def test_backward_against_finite_differences_of_the_float64_layer():
    """Brute force on a tiny layer.  L = sum(G * layer(x)) in float64; its gradients by central differences.
    What the unit-scaled backward pass must return differs from the true gradient only by fixed ratios:
      branch input gradient: (beta_x1 beta_g beta_x2) / (alpha_1 alpha_g alpha_2) = beta_g / alpha_g
                             (the matmul factors cancel: beta_x1 = alpha_2 = f^-1/2, beta_x2 = alpha_1 = d^-1/2),
      grad_W2: beta_w2 / alpha_2 = sqrt(f / T) and no sqrt(tau);  grad_W1: sqrt(f / T) beta_g / alpha_g, no sqrt(tau);
      layer input gradient: sqrt(1-tau) g + sqrt(tau) * (branch input gradient).
    The oracle's FP16 roundings leave about 1e-3 of a unit-scale value."""
    T, d, f, tau = 16, 16, 32, 0.3
    X16, W1_16, W2_16, G16 = synth.ffn_inputs(T, d, f, seed=83)
    ag, bg = (float(v) for v in oracle.gelu_scales())
    X, W1, W2, G = (a.astype(np.float64) for a in (X16, W1_16, W2_16, G16))
    loss = lambda: float(np.sum(G * _f64_layer(X, W1, W2, tau, ag)))
    gX, gW1, gW2 = _fd_grad(loss, X), _fd_grad(loss, W1), _fd_grad(loss, W2)
    fw = oracle.ffn_res_fwd(X16, W1_16, W2_16, tau, False)
    bw = oracle.ffn_res_bwd(X16, W1_16, W2_16, G16, fw, tau, False)
    skip, branch = math.sqrt(1 - tau), math.sqrt(tau)
    assert np.allclose(fw["Out"].astype(np.float64), _f64_layer(X, W1, W2, tau, ag), atol=6e-3)
    branch_true = (gX - skip * G) / branch                               # J_branch^T G
    assert np.allclose(bw["dX"].astype(np.float64), bg / ag * branch_true, atol=8e-3)
    assert np.allclose(bw["dXin"].astype(np.float64), skip * G + branch * (bg / ag) * branch_true, atol=8e-3)
    assert np.allclose(bw["dW2"].astype(np.float64), math.sqrt(f / T) * gW2 / branch, atol=8e-3)
    assert np.allclose(bw["dW1"].astype(np.float64), math.sqrt(f / T) * (bg / ag) * gW1 / branch, atol=8e-3)
    # a transposed operand or a swapped fan_in / fan_out would be far outside: the gradients are O(1)
    assert np.std(bw["dW1"].astype(np.float64)) > 0.5 and np.std(bw["dXin"].astype(np.float64)) > 0.5
