"""Pins for the oracle's batched matmuls and the unit-scaled attention built from them (CPU only): numpy's float64
matmul on every transposition, torch's float64 attention and its autograd (with the unit-scaling factors undone),
the factors as Table A.2's rule gives them, and the scale of every tensor for unit-normal inputs."""
import numpy as np
import torch

import oracle
import synth


def _f16(a):
    return np.asarray(a, np.float64).astype(np.float16)


def _close(a, ref, ulps=1.0):
    a, ref = a.astype(np.float64), np.asarray(ref, np.float64)
    return bool(np.all(np.abs(a - ref) <= ulps * 2.0 ** -10 * np.abs(ref) + 1e-6))


def test_batched_matmul_every_transposition_against_numpy():
    h, M, N, K = 3, 20, 12, 28
    A = synth.normal(95, 1, (h, M, K)); B = synth.normal(95, 2, (h, K, N))
    Ad, Bd = A.astype(np.float64), B.astype(np.float64)
    C = oracle.matmul_batched(A, B, 0.25)
    assert C.shape == (h, M, N) and np.array_equal(C, _f16(0.25 * Ad @ Bd))
    Bt = np.ascontiguousarray(B.transpose(0, 2, 1))                   # [h, N, K]
    assert np.array_equal(oracle.matmul_batched(A, Bt, 0.25, trans_b=True), C)
    At = np.ascontiguousarray(A.transpose(0, 2, 1))                   # [h, K, M]
    assert np.array_equal(oracle.matmul_batched(At, B, 0.25, trans_a=True), C)
    # the slices are independent: permuting the batch permutes the result
    perm = [2, 0, 1]
    assert np.array_equal(oracle.matmul_batched(A[perm], B[perm], 0.25), C[perm])


def test_attention_factors_follow_table_a2():
    c = oracle.attention_scales(512, 64)
    assert c["a_scores"] == np.float32(64 ** -0.5)                    # App. F: the familiar 1/sqrt(d) ...
    assert c["b_q"] == c["b_k"] == np.float32(512 ** -0.5)            # ... but the gradients reduce over s, not d
    assert c["a_soft"] == c["b_soft"] == 512
    assert c["a_out"] == np.float32(512 ** -0.5) and c["b_p"] == np.float32(64 ** -0.5) and c["b_v"] == np.float32(512 ** -0.5)


def test_attention_against_float64_torch_and_autograd():
    h, s, d = 2, 48, 16
    Q, K, V, dO = (synth.normal(96, i, (h, s, d)) for i in (1, 2, 3, 4))
    fw = oracle.attention_fwd(Q, K, V)
    bw = oracle.attention_bwd(Q, K, V, dO, fw)
    t = lambda a: torch.tensor(a.astype(np.float64), requires_grad=True)
    q, k, v = t(Q), t(K), t(V)
    a = q @ k.transpose(1, 2) / d ** 0.5
    p = torch.softmax(a, dim=-1)
    o = p @ v
    # forward: A as is; P = s * softmax; O = s^-1/2 * (s p) v = s^1/2 * (p v)
    assert _close(fw["A"], a.detach().numpy())
    assert _close(fw["P"], s * p.detach().numpy(), 3)                 # p from the rounded A
    # O sums s rounded products with cancellation: absolute agreement at the level of the roundings of A and P
    assert np.allclose(fw["O"].astype(np.float64), s ** 0.5 * o.detach().numpy(), rtol=4e-3, atol=4e-3)
    # backward, op by op, each compared with autograd of the matching unscaled op on the oracle's own stored inputs
    Pd, Ad = fw["P"].astype(np.float64), fw["A"].astype(np.float64)
    dOd = dO.astype(np.float64)
    assert _close(bw["dV"], s ** -0.5 * Pd.transpose(0, 2, 1) @ dOd)
    assert _close(bw["dP"], d ** -0.5 * dOd @ V.astype(np.float64).transpose(0, 2, 1))
    at = torch.tensor(Ad, requires_grad=True)
    (torch.softmax(at, dim=-1) * torch.tensor(bw["dP"].astype(np.float64))).sum().backward()
    assert _close(bw["dA"], s * at.grad.numpy(), 2)
    dAd = bw["dA"].astype(np.float64)
    assert _close(bw["dQ"], s ** -0.5 * dAd @ K.astype(np.float64))
    assert _close(bw["dK"], s ** -0.5 * dAd.transpose(0, 2, 1) @ Q.astype(np.float64))
    # and the whole chain against autograd of the unscaled attention, the factors undone: along the path to V the
    # unit-scaled backward differs from the true gradient of the unit-scaled forward by beta_v / alpha_out = 1
    (o * torch.tensor(dOd)).sum().backward()
    assert np.allclose(bw["dV"].astype(np.float64), s ** 0.5 * v.grad.numpy(), rtol=0.02, atol=0.02)
    # to Q: dP (d^-1/2 instead of a_out = s^-1/2 ... relative to autograd's dP = dO v^T), softmax (s instead of 1/..)
    ratio = (d ** -0.5) * s * (s ** -0.5) / (d ** -0.5)               # b_p * b_soft * b_q over autograd's 1 * 1 * d^-1/2
    assert np.allclose(bw["dQ"].astype(np.float64), ratio * q.grad.numpy(), rtol=0.03, atol=0.03)
    assert np.allclose(bw["dK"].astype(np.float64), ratio * k.grad.numpy(), rtol=0.03, atol=0.03)


def test_scale_of_every_tensor_for_unit_normal_inputs():
    h, s, d = 4, 256, 64
    Q, K, V, dO = (synth.normal(97, i, (h, s, d)) for i in (1, 2, 3, 4))
    fw = oracle.attention_fwd(Q, K, V)
    bw = oracle.attention_bwd(Q, K, V, dO, fw)
    sd = lambda a: float(a.astype(np.float64).std())
    assert abs(sd(fw["A"]) - 1.0) < 0.03                              # the 1/sqrt(d) of App. F
    assert abs(float(fw["P"].astype(np.float64).mean()) - 1.0) < 1e-3  # about a vector of ones
    # O = s^-1/2 sum_j (s p_j) v_j: variance = mean (s p)^2 = e for unit-normal scores (the paper's uniform-p assumption gives 1)
    assert abs(sd(fw["O"]) ** 2 - np.e) < 0.5
    assert abs(sd(bw["dP"]) - 1.0) < 0.03
    assert abs(sd(bw["dV"]) ** 2 - np.e) < 0.5
    assert 1.0 < sd(bw["dA"]) < 2.2 and 1.0 < sd(bw["dQ"]) < 2.5 and 1.0 < sd(bw["dK"]) < 2.5   # within a binade or so of 1
