"""GPU parity for the batched scaled matmul (us_matmul_batched) and the unit-scaled attention composed of it and the
scaled softmax (us_attention_fwd / us_attention_bwd), stage by stage against the oracle on the GPU's own stored inputs."""
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


def _batched(A, B, scale, trans_a=False, trans_b=False, a_dt=us.F16, b_dt=us.F16, out=np.float16):
    batch = A.shape[0]
    M = A.shape[2] if trans_a else A.shape[1]
    K = A.shape[1] if trans_a else A.shape[2]
    N = B.shape[1] if trans_b else B.shape[2]
    tA, tB, tC = to_dev(A), to_dev(B), empty((batch, M, N), out)
    us.matmul_batched(ptr(tA), ptr(tB), ptr(tC), batch, M, N, K, trans_a, trans_b, a_dt, b_dt, us.F16 if out == np.float16 else us.F32,
                      scale, stream())
    return to_np(tC)


# (batch, M, N, K): ragged K (register-staged kernel), ragged tile edges, attention scores, attention output, large tiles
SHAPES = [(3, 48, 80, 112), (5, 272, 144, 256), (16, 512, 512, 64), (16, 512, 64, 512), (24, 1024, 1024, 128)]


@pytest.mark.parametrize("mode", ["nn", "nt", "tn"])
@pytest.mark.parametrize("shape", SHAPES)
def test_matmul_batched_fp16(shape, mode):
    batch, M, N, K = shape
    ta, tb = mode == "tn", mode == "nt"
    A = synth.normal(98, 1, (batch, K, M) if ta else (batch, M, K))
    B = synth.normal(98, 2, (batch, N, K) if tb else (batch, K, N))
    scale = float(K) ** -0.5
    C = _batched(A, B, scale, ta, tb)
    sel = range(batch) if batch * M * N * K < 3e9 else [0, batch // 2, batch - 1]
    for i in sel:
        ref = O.matmul_batched(A[i:i + 1], B[i:i + 1], scale, ta, tb)[0]
        assert_close(C[i], ref, f"{mode} {shape} item {i}")


@pytest.mark.parametrize("mode", ["nn", "nt", "tn"])
def test_matmul_batched_fp8_pairs_and_fp32_output(mode):
    batch, M, N, K = 4, 272, 144, 256
    ta, tb = mode == "tn", mode == "nt"
    A16 = synth.normal(99, 1, (batch, K, M) if ta else (batch, M, K))
    B16 = synth.normal(99, 2, (batch, N, K) if tb else (batch, K, N))
    fa, fb = {"nn": (O.E4M3, O.E4M3), "nt": (O.E5M2, O.E4M3), "tn": (O.E4M3, O.E5M2)}[mode]
    A8, B8 = O.cast_fp8(A16, fa)[0], O.cast_fp8(B16, fb)[0]
    C = _batched(A8, B8, 1 / 16, ta, tb, a_dt=fa, b_dt=fb, out=np.float32)
    ref = O.matmul_batched(A8, B8, 1 / 16, ta, tb, fa, fb, O.F32)
    assert_close(C, ref, mode, fp8=True)


def test_matmul_batched_exact_integers_and_independent_items():
    batch, M, N, K = 6, 144, 80, 192
    A = synth.small_ints(100, 1, (batch, M, K))
    B = synth.small_ints(100, 2, (batch, K, N))
    C = _batched(A, B, 0.125)
    exact = (0.125 * A.astype(np.float64) @ B.astype(np.float64)).astype(np.float16)
    assert np.array_equal(_bits(C), _bits(exact))
    perm = [3, 0, 5, 1, 4, 2]
    assert np.array_equal(_bits(_batched(A[perm], B[perm], 0.125)), _bits(C[perm]))


def test_a_batch_of_one_is_the_plain_matmul():
    M, N, K = 272, 400, 256
    A = synth.normal(102, 1, (1, M, K)); B = synth.normal(102, 2, (1, K, N))
    C = _batched(A, B, 1 / 16)
    tA, tB, tY = to_dev(A[0]), to_dev(B[0]), empty((M, N), np.float16)
    us.linear_fwd(ptr(tA), ptr(tB), ptr(tY), M, K, N, us.F16, us.F16, us.F16, 1 / 16, us.EPI_NONE, 0.0, None, None, None, 0, stream())
    assert np.array_equal(_bits(C[0]), _bits(to_np(tY)))


def test_zero_reduction_length_and_special_values():
    C = _batched(np.zeros((3, 32, 0), np.float16), np.zeros((3, 0, 48), np.float16), 1.0)
    assert C.shape == (3, 32, 48) and not C.any()
    A = synth.normal(103, 1, (2, 48, 64)); B = synth.normal(103, 2, (2, 64, 32))
    A[1, 5, 7] = np.nan
    A[0, 3, :] = 0; A[0, 3, 0] = np.inf; B[0, 0, :] = 1.0
    C = _batched(A, B, 1.0)
    assert np.all(np.isnan(C[1, 5])) and np.isfinite(C[1, 4]).all()
    assert np.all(np.isinf(C[0, 3])) and np.isfinite(C[0, 2]).all()


class Attn:
    def __init__(self, heads, s, d, seed, on_device=False):
        self.heads, self.s, self.d = heads, s, d
        if on_device:
            Q, K, V, dO = (synth.normal_on_device(seed, i, (heads, s, d)) for i in (1, 2, 3, 4))
        else:
            Q, K, V, dO = (to_dev(synth.normal(seed, i, (heads, s, d))) for i in (1, 2, 3, 4))
        e = lambda *shape: torch.empty(shape, dtype=torch.float16, device=DEV)
        t = dict(Q=Q, K=K, V=V, dO=dO, A=e(heads, s, s), P=e(heads, s, s), O=e(heads, s, d), dP=e(heads, s, s), dA=e(heads, s, s),
                 dQ=e(heads, s, d), dK=e(heads, s, d), dV=e(heads, s, d))
        st = stream()
        us.attention_fwd(ptr(Q), ptr(K), ptr(V), ptr(t["A"]), ptr(t["P"]), ptr(t["O"]), heads, s, d, st)
        us.attention_bwd(ptr(Q), ptr(K), ptr(V), ptr(t["A"]), ptr(t["P"]), ptr(dO), ptr(t["dP"]), ptr(t["dA"]), ptr(t["dQ"]), ptr(t["dK"]),
                         ptr(t["dV"]), heads, s, d, st)
        torch.cuda.synchronize()
        self.t = t

    def head(self, name, h):
        return self.t[name][h:h + 1].cpu().numpy()


def _soft_close(gpu, ref):
    g, r = gpu.astype(np.float64), ref.astype(np.float64)
    assert np.all(np.abs(g - r) <= 2.0 ** -10 * np.abs(r) + 1e-6)


def check_heads(run, heads):
    s, d = run.s, run.d
    c = O.attention_scales(s, d)
    for h in heads:
        g = {k: run.head(k, h) for k in run.t}
        assert_close(g["A"], O.matmul_batched(g["Q"], g["K"], c["a_scores"], trans_b=True), "A")
        _soft_close(g["P"][0], O.softmax_fwd(g["A"][0], c["a_soft"]))
        assert_close(g["O"], O.matmul_batched(g["P"], g["V"], c["a_out"]), "O")
        assert_close(g["dV"], O.matmul_batched(g["P"], g["dO"], c["b_v"], trans_a=True), "dV")
        assert_close(g["dP"], O.matmul_batched(g["dO"], g["V"], c["b_p"], trans_b=True), "dP")
        _soft_close(g["dA"][0], O.softmax_bwd(g["A"][0], g["dP"][0], c["b_soft"]))
        assert_close(g["dQ"], O.matmul_batched(g["dA"], g["K"], c["b_q"]), "dQ")
        assert_close(g["dK"], O.matmul_batched(g["dA"], g["Q"], c["b_k"], trans_a=True), "dK")


@pytest.mark.parametrize("shape", [(1, 16, 16), (3, 80, 48), (2, 272, 64), (5, 128, 128)])
def test_attention_small_shapes_every_head(shape):
    heads, s, d = shape
    check_heads(Attn(heads, s, d, 101), range(heads))


def test_attention_at_bert_large_size_sampled_heads():
    heads, s, d = 16 * 16, 512, 64                    # 16 sequences x 16 heads, 512 tokens, head size 64
    run = Attn(heads, s, d, 20230315, on_device=True)
    check_heads(run, [0, 77, 255])
    t = run.t
    assert abs(float(t["A"].float().std()) - 1.0) < 0.02 and abs(float(t["P"].float().mean()) - 1.0) < 1e-3
    assert abs(float(t["O"].float().var()) - np.e) < 0.4 and abs(float(t["dP"].float().std()) - 1.0) < 0.02
