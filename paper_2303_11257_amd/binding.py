"""ctypes binding of the C ABI declared in ``include/us.h``.

Argument marshalling only: every function takes raw device addresses (``tensor.data_ptr()``) and a
HIP stream handle, forwards them unchanged and raises :class:`UsError` on a non-zero status.  There
is no fallback: if the shared library has not been built, importing it fails.
"""
from __future__ import annotations

import ctypes
import os

F32, F16, E4M3, E5M2 = 0, 1, 2, 3
EPI_NONE, EPI_GELU, EPI_GELU_GRAD, EPI_RESIDUAL = 0, 1, 2, 3
EPI_ACT_RELU, EPI_ACT_TANH, EPI_ACT_SIGMOID = 0x10, 0x20, 0x30   # OR-ed onto EPI_GELU / EPI_GELU_GRAD
ACT_GELU, ACT_RELU, ACT_TANH, ACT_SIGMOID = 0, 1, 2, 3
EPI_TABLES_READY = 0x100            # flag for EPI_GELU / EPI_GELU_GRAD: tables prebuilt by gelu_tables()
FFN_FP8, FFN_TABLES_READY = 1, 2    # mode bits of ffn_fwd / ffn_bwd
TABLE_AREA_BYTES = 256 * 1024
HIST_BINS = 35
STATUS = {0: "US_OK", 1: "US_ERR_NULL", 2: "US_ERR_SHAPE", 3: "US_ERR_ALIGN", 4: "US_ERR_DTYPE",
          5: "US_ERR_WORKSPACE", 6: "US_ERR_LAUNCH", 7: "US_ERR_VALUE"}

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libus_mi355x.so")
_lib = None


class UsError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {STATUS.get(status, status)} ({status_string(status)})")


def library_path() -> str:
    return _LIB_PATH


def lib() -> ctypes.CDLL:
    """Loads libus_mi355x.so (built by ``paper_2303_11257_amd.build``); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(f"{_LIB_PATH} not built: run `python -m paper_2303_11257_amd.build`")
    L = ctypes.CDLL(_LIB_PATH)
    vp, i, l, f, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_long, ctypes.c_float, ctypes.c_size_t
    fp = ctypes.POINTER(ctypes.c_float)
    L.us_status_string.argtypes = [i]
    L.us_status_string.restype = ctypes.c_char_p
    L.us_last_launch.argtypes = []
    L.us_last_launch.restype = ctypes.c_char_p
    L.us_linear_scales.argtypes = [l, l, l, i, fp, fp, fp]
    L.us_cast_fp8.argtypes = [vp, i, vp, i, sz, f, vp, vp]
    L.us_cast_fp8_batch.argtypes = [i, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(sz), ctypes.POINTER(i), vp]
    L.us_linear_fwd.argtypes = [vp, vp, vp, l, l, l, i, i, i, f, i, f, vp, vp, vp, sz, vp]
    L.us_linear_bwd.argtypes = [vp, vp, vp, vp, vp, l, l, l, i, i, i, i, f, f, i, f, vp, vp, vp, sz, vp]
    L.us_workspace_bytes.argtypes = [l, l, l]
    L.us_linear_bwd_noalloc.argtypes = [vp, vp, vp, vp, vp, l, l, l, i, i, i, i, f, f, i, f, vp, vp, vp]
    L.us_noalloc_scratch_bytes.argtypes = []
    L.us_noalloc_scratch_bytes.restype = sz
    L.us_gelu_tables.argtypes = [vp, sz, f, f, vp]
    L.us_weighted_add.argtypes = [vp, vp, vp, sz, i, f, f, vp]
    L.us_layer_norm_fwd.argtypes = [vp, vp, vp, vp, l, l, f, vp]
    L.us_layer_norm_bwd.argtypes = [vp, vp, vp, vp, vp, vp, l, l, f, f, vp, sz, vp]
    L.us_layer_norm_workspace_bytes.argtypes = [l, l]
    L.us_layer_norm_workspace_bytes.restype = sz
    L.us_exponent_histogram.argtypes = [vp, i, sz, vp, vp]
    L.us_cast_snr.argtypes = [vp, i, sz, i, f, vp, vp]
    L.us_act_fwd.argtypes = [vp, vp, sz, i, i, f, f, vp]
    L.us_act_bwd.argtypes = [vp, vp, vp, sz, i, i, f, f, vp]
    L.us_ffn_res_fwd.argtypes = [vp] * 7 + [l, l, l, f, i, vp, sz, vp]
    L.us_ffn_res_bwd.argtypes = [vp] * 12 + [l, l, l, f, i, vp, sz, vp]
    L.us_workspace_bytes.restype = sz
    L.us_gelu_fwd.argtypes = [vp, vp, sz, i, f, vp]
    L.us_gelu_bwd.argtypes = [vp, vp, vp, sz, i, f, vp]
    L.us_ffn_fwd.argtypes = [vp, vp, vp, vp, vp, vp, l, l, l, i, vp, sz, vp]
    L.us_ffn_bwd.argtypes = [vp] * 11 + [l, l, l, i, vp, sz, vp]
    L.us_ffn_workspace_bytes.argtypes = [l, l, l]
    L.us_ffn_workspace_bytes.restype = sz
    L.us_matmul_batched.argtypes = [vp, vp, vp, l, l, l, l, i, i, i, i, i, f, vp]
    L.us_attention_fwd.argtypes = [vp] * 6 + [l, l, l, vp]
    L.us_attention_bwd.argtypes = [vp] * 11 + [l, l, l, vp]
    L.us_sum_fwd.argtypes = [vp, vp, l, l, f, vp]
    L.us_sum_bwd.argtypes = [vp, vp, l, l, f, vp]
    L.us_softmax_fwd.argtypes = [vp, vp, l, l, f, f, vp]
    L.us_softmax_bwd.argtypes = [vp, vp, vp, l, l, f, f, vp]
    L.us_softmax_xent.argtypes = [vp, vp, vp, vp, l, l, f, f, vp]
    L.us_linear_bias_fwd.argtypes = [vp, vp, vp, vp, l, l, l, i, i, i, f, i, f, vp, vp, vp, sz, vp]
    L.us_bias_grad.argtypes = [vp, i, vp, l, l, f, vp, sz, vp]
    L.us_bias_grad_workspace_bytes.argtypes = [l, l]
    L.us_bias_grad_workspace_bytes.restype = sz
    L.us_ffn_bias_fwd.argtypes = [vp] * 8 + [l, l, l, i, vp, sz, vp]
    L.us_ffn_bias_bwd.argtypes = [vp] * 14 + [l, l, l, i, vp, sz, vp]
    L.us_ffn_bias_workspace_bytes.argtypes = [l, l, l]
    L.us_ffn_bias_workspace_bytes.restype = sz
    for name in ("us_linear_scales", "us_cast_fp8", "us_cast_fp8_batch", "us_linear_fwd", "us_linear_bwd", "us_linear_bwd_noalloc", "us_gelu_fwd", "us_gelu_bwd",
                 "us_gelu_tables", "us_ffn_fwd", "us_ffn_bwd", "us_weighted_add", "us_ffn_res_fwd", "us_ffn_res_bwd", "us_act_fwd", "us_act_bwd", "us_layer_norm_fwd", "us_layer_norm_bwd", "us_exponent_histogram", "us_cast_snr",
                 "us_linear_bias_fwd", "us_bias_grad", "us_ffn_bias_fwd", "us_ffn_bias_bwd", "us_softmax_fwd", "us_softmax_bwd",
                 "us_softmax_xent", "us_matmul_batched", "us_attention_fwd", "us_attention_bwd", "us_sum_fwd", "us_sum_bwd"):
        getattr(L, name).restype = i
    _lib = L
    return L


def last_launch() -> str:
    """Which matmul kernels this thread's most recent matmul call enqueued (see us_last_launch in include/us.h)."""
    return lib().us_last_launch().decode()


def status_string(status: int) -> str:
    return lib().us_status_string(status).decode()


def _check(status: int, where: str) -> None:
    if status != 0:
        raise UsError(status, where)


def linear_scales(b: int, m: int, n: int, mode: int = 0):
    a, bx, bw = ctypes.c_float(), ctypes.c_float(), ctypes.c_float()
    _check(lib().us_linear_scales(b, m, n, mode, ctypes.byref(a), ctypes.byref(bx), ctypes.byref(bw)), "us_linear_scales")
    return a.value, bx.value, bw.value


def cast_fp8(src, src_dt, dst, dst_dt, n, scale=1.0, stats=None, stream=None):
    _check(lib().us_cast_fp8(src, src_dt, dst, dst_dt, n, scale, stats, stream), "us_cast_fp8")


def cast_fp8_batch(srcs, dsts, ns, dst_dts, stream=None):
    """One launch for several FP16 tensors: sequences of device addresses, element counts and FP8 types."""
    k = len(srcs)
    A = lambda T, vals: (T * k)(*vals)
    _check(lib().us_cast_fp8_batch(k, A(ctypes.c_void_p, srcs), A(ctypes.c_void_p, dsts), A(ctypes.c_size_t, ns),
                                   A(ctypes.c_int, dst_dts), stream), "us_cast_fp8_batch")


def linear_fwd(X, W, Y, b, m, n, x_dt, w_dt, y_dt=F16, alpha=0.0, epi=EPI_NONE, epi_scale=0.0, aux16=None, aux8=None,
               workspace=None, workspace_bytes=0, stream=None):
    _check(lib().us_linear_fwd(X, W, Y, b, m, n, x_dt, w_dt, y_dt, alpha, epi, epi_scale, aux16, aux8, workspace,
                               workspace_bytes, stream), "us_linear_fwd")


def linear_bwd(X, W, G, dX, dW, b, m, n, x_dt, w_dt, g_dt, out_dt=F16, beta_x=0.0, beta_w=0.0, epi=EPI_NONE,
               epi_scale=0.0, Zpre=None, aux8=None, workspace=None, workspace_bytes=0, stream=None):
    _check(lib().us_linear_bwd(X, W, G, dX, dW, b, m, n, x_dt, w_dt, g_dt, out_dt, beta_x, beta_w, epi, epi_scale, Zpre,
                               aux8, workspace, workspace_bytes, stream), "us_linear_bwd")


def linear_bwd_noalloc(X, W, G, dX, dW, b, m, n, x_dt, w_dt, g_dt, out_dt=F16, beta_x=0.0, beta_w=0.0, epi=EPI_NONE,
                       epi_scale=0.0, Zpre=None, aux8=None, stream=None):
    _check(lib().us_linear_bwd_noalloc(X, W, G, dX, dW, b, m, n, x_dt, w_dt, g_dt, out_dt, beta_x, beta_w, epi, epi_scale, Zpre,
                                       aux8, stream), "us_linear_bwd_noalloc")


def noalloc_scratch_bytes() -> int:
    return int(lib().us_noalloc_scratch_bytes())


def workspace_bytes(b: int, m: int, n: int) -> int:
    return int(lib().us_workspace_bytes(b, m, n))


def gelu_tables(workspace, workspace_bytes, alpha_g=0.0, beta_g=0.0, stream=None):
    _check(lib().us_gelu_tables(workspace, workspace_bytes, alpha_g, beta_g, stream), "us_gelu_tables")


def gelu_fwd(z, h, n, dt=F16, alpha_g=0.0, stream=None):
    _check(lib().us_gelu_fwd(z, h, n, dt, alpha_g, stream), "us_gelu_fwd")


def gelu_bwd(z, gh, gz, n, dt=F16, beta_g=0.0, stream=None):
    _check(lib().us_gelu_bwd(z, gh, gz, n, dt, beta_g, stream), "us_gelu_bwd")


def ffn_fwd(X, W1, W2, Z, H, Y, T, d, f, mode, workspace=None, workspace_bytes=0, stream=None):
    """mode: FFN_FP8 (or True) for FP8 operands, optionally | FFN_TABLES_READY."""
    _check(lib().us_ffn_fwd(X, W1, W2, Z, H, Y, T, d, f, int(mode), workspace, workspace_bytes, stream), "us_ffn_fwd")


def ffn_bwd(X, W1, W2, Z, H, G, dZ16, dZ8, dX, dW1, dW2, T, d, f, mode, workspace=None, workspace_bytes=0, stream=None):
    _check(lib().us_ffn_bwd(X, W1, W2, Z, H, G, dZ16, dZ8, dX, dW1, dW2, T, d, f, int(mode), workspace, workspace_bytes,
                            stream), "us_ffn_bwd")


def ffn_workspace_bytes(T: int, d: int, f: int) -> int:
    return int(lib().us_ffn_workspace_bytes(T, d, f))


def weighted_add(a, b, out, n, dt=F16, ca=1.0, cb=1.0, stream=None):
    _check(lib().us_weighted_add(a, b, out, n, dt, ca, cb, stream), "us_weighted_add")


def ffn_res_fwd(Xskip, X, W1, W2, Z, H, Out, T, d, f, tau, mode, workspace=None, workspace_bytes=0, stream=None):
    _check(lib().us_ffn_res_fwd(Xskip, X, W1, W2, Z, H, Out, T, d, f, tau, int(mode), workspace, workspace_bytes, stream),
           "us_ffn_res_fwd")


def ffn_res_bwd(X, W1, W2, Z, H, Gskip, G, dZ16, dZ8, dXin, dW1, dW2, T, d, f, tau, mode, workspace=None, workspace_bytes=0,
                stream=None):
    _check(lib().us_ffn_res_bwd(X, W1, W2, Z, H, Gskip, G, dZ16, dZ8, dXin, dW1, dW2, T, d, f, tau, int(mode), workspace,
                                workspace_bytes, stream), "us_ffn_res_bwd")


def linear_bias_fwd(X, W, bias, Y, b, m, n, x_dt, w_dt, y_dt=F16, alpha=0.0, epi=EPI_NONE, epi_scale=0.0, aux16=None, aux8=None,
                    workspace=None, workspace_bytes=0, stream=None):
    _check(lib().us_linear_bias_fwd(X, W, bias, Y, b, m, n, x_dt, w_dt, y_dt, alpha, epi, epi_scale, aux16, aux8, workspace,
                                    workspace_bytes, stream), "us_linear_bias_fwd")


def bias_grad(G, g_dt, dc, b, n, beta_c=0.0, workspace=None, workspace_bytes=0, stream=None):
    _check(lib().us_bias_grad(G, g_dt, dc, b, n, beta_c, workspace, workspace_bytes, stream), "us_bias_grad")


def bias_grad_workspace_bytes(b: int, n: int) -> int:
    return int(lib().us_bias_grad_workspace_bytes(b, n))


def ffn_bias_fwd(X, W1, b1, W2, b2, Z, H, Y, T, d, f, mode, workspace=None, workspace_bytes=0, stream=None):
    _check(lib().us_ffn_bias_fwd(X, W1, b1, W2, b2, Z, H, Y, T, d, f, int(mode), workspace, workspace_bytes, stream),
           "us_ffn_bias_fwd")


def ffn_bias_bwd(X, W1, W2, Z, H, G, G16, dZ16, dZ8, dX, dW1, dW2, db1, db2, T, d, f, mode, workspace=None, workspace_bytes=0,
                 stream=None):
    _check(lib().us_ffn_bias_bwd(X, W1, W2, Z, H, G, G16, dZ16, dZ8, dX, dW1, dW2, db1, db2, T, d, f, int(mode), workspace,
                                 workspace_bytes, stream), "us_ffn_bias_bwd")


def ffn_bias_workspace_bytes(T: int, d: int, f: int) -> int:
    return int(lib().us_ffn_bias_workspace_bytes(T, d, f))


def matmul_batched(A, B, C, batch, M, N, K, trans_a, trans_b, a_dt, b_dt, c_dt, scale, stream=None):
    _check(lib().us_matmul_batched(A, B, C, batch, M, N, K, int(trans_a), int(trans_b), a_dt, b_dt, c_dt, scale, stream),
           "us_matmul_batched")


def attention_fwd(Q, K, V, A, P, O, heads, s, d, stream=None):
    _check(lib().us_attention_fwd(Q, K, V, A, P, O, heads, s, d, stream), "us_attention_fwd")


def attention_bwd(Q, K, V, A, P, dO, dP, dA, dQ, dK, dV, heads, s, d, stream=None):
    _check(lib().us_attention_bwd(Q, K, V, A, P, dO, dP, dA, dQ, dK, dV, heads, s, d, stream), "us_attention_bwd")


def sum_fwd(X, Y, rows, n, alpha=0.0, stream=None):
    _check(lib().us_sum_fwd(X, Y, rows, n, alpha, stream), "us_sum_fwd")


def sum_bwd(G, dX, rows, n, beta=0.0, stream=None):
    _check(lib().us_sum_bwd(G, dX, rows, n, beta, stream), "us_sum_bwd")


def softmax_fwd(X, Y, rows, s, s1=0.0, alpha=0.0, stream=None):
    _check(lib().us_softmax_fwd(X, Y, rows, s, s1, alpha, stream), "us_softmax_fwd")


def softmax_bwd(X, G, dX, rows, s, s1=0.0, beta=0.0, stream=None):
    _check(lib().us_softmax_bwd(X, G, dX, rows, s, s1, beta, stream), "us_softmax_bwd")


def softmax_xent(X, target, loss, dX, rows, s, s1=0.0, beta=0.0, stream=None):
    _check(lib().us_softmax_xent(X, target, loss, dX, rows, s, s1, beta, stream), "us_softmax_xent")


def act_fwd(z, h, n, dt=F16, kind=ACT_GELU, s1=0.0, scale=0.0, stream=None):
    _check(lib().us_act_fwd(z, h, n, dt, kind, s1, scale, stream), "us_act_fwd")


def act_bwd(z, gh, gz, n, dt=F16, kind=ACT_GELU, s1=0.0, scale=0.0, stream=None):
    _check(lib().us_act_bwd(z, gh, gz, n, dt, kind, s1, scale, stream), "us_act_bwd")


def layer_norm_fwd(X, w, c, Y, b, n, eps=0.0, stream=None):
    _check(lib().us_layer_norm_fwd(X, w, c, Y, b, n, eps, stream), "us_layer_norm_fwd")


def layer_norm_bwd(X, w, G, dX, dw, dc, b, n, eps=0.0, beta_wc=0.0, workspace=None, workspace_bytes=0, stream=None):
    _check(lib().us_layer_norm_bwd(X, w, G, dX, dw, dc, b, n, eps, beta_wc, workspace, workspace_bytes, stream), "us_layer_norm_bwd")


def layer_norm_workspace_bytes(b: int, n: int) -> int:
    return int(lib().us_layer_norm_workspace_bytes(b, n))


def exponent_histogram(src, src_dt, n, hist, stream=None):
    """hist: device pointer to HIST_BINS uint64 counters (added to)."""
    _check(lib().us_exponent_histogram(src, src_dt, n, hist, stream), "us_exponent_histogram")


def cast_snr(src, src_dt, n, dst_dt, scale, sums, stream=None):
    """sums: device pointer to two float64 (added to): sum x^2 and sum (q(x*scale)/scale - x)^2."""
    _check(lib().us_cast_snr(src, src_dt, n, dst_dt, scale, sums, stream), "us_cast_snr")
