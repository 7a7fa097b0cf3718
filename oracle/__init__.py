"""CPU oracle for the unit-scaled linear / FFN hot path -- TEST INFRASTRUCTURE ONLY.

Thin numpy front-end over ``us_oracle.c`` (plain C, double arithmetic, index-order sums; see the
header of that file for the passages of the paper each function follows).  Only the tests, the
smoke check and the benchmark's ``cpu_baseline`` leg may import this package; the HIP library
and its Python binding never do, and this package imports nothing from them.

Array conventions: FP32 -> ``np.float32``, FP16 -> ``np.float16``, FP8 -> ``np.uint8`` codes
(OCP E4M3 / E5M2 = rows "E4 (b)" / "E5 (b)" of Table A.1).  All matrices are row-major:
X[b,m], W[m,n], G[b,n].
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess

import numpy as np

F32, F16, E4M3, E5M2 = 0, 1, 2, 3

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "us_oracle.c")
_LIB = os.path.join(_HERE, "libus_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile us_oracle.c with gcc (-O2, OpenMP, no FP contraction). Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    lib = ctypes.CDLL(build())
    vp, i, l, f, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_long, ctypes.c_float, ctypes.c_size_t
    lib.uso_decode_bits.argtypes = [ctypes.c_uint32, i]
    lib.uso_decode_bits.restype = ctypes.c_double
    lib.uso_encode_f64.argtypes = [ctypes.c_double, i, i]
    lib.uso_encode_f64.restype = ctypes.c_uint32
    lib.uso_decode.argtypes = [vp, i, sz, vp]
    lib.uso_decode.restype = None
    lib.uso_encode.argtypes = [vp, sz, i, i, vp]
    lib.uso_encode.restype = None
    lib.uso_cast_fp8.argtypes = [vp, i, vp, i, sz, f, vp]
    lib.uso_cast_fp8.restype = None
    for name in ("uso_linear_fwd", "uso_linear_bwd_dx", "uso_linear_bwd_dw"):
        fn = getattr(lib, name)
        fn.argtypes = [vp, i, vp, i, vp, i, l, l, l, f]
        fn.restype = i
    lib.uso_linear_bias_fwd.argtypes = [vp, i, vp, i, vp, vp, i, l, l, l, f]
    lib.uso_linear_bias_fwd.restype = i
    lib.uso_bias_grad.argtypes = [vp, i, vp, i, l, l, f]
    lib.uso_bias_grad.restype = None
    lib.uso_sum_fwd.argtypes = [vp, vp, l, l, f]
    lib.uso_sum_fwd.restype = None
    lib.uso_sum_bwd.argtypes = [vp, vp, l, l, f]
    lib.uso_sum_bwd.restype = None
    lib.uso_softmax_fwd.argtypes = [vp, vp, l, l, f, f]
    lib.uso_softmax_fwd.restype = None
    lib.uso_softmax_bwd.argtypes = [vp, vp, vp, l, l, f, f]
    lib.uso_softmax_bwd.restype = None
    lib.uso_softmax_xent.argtypes = [vp, vp, vp, vp, l, l, f, f]
    lib.uso_softmax_xent.restype = None
    lib.uso_gelu_fwd.argtypes = [vp, vp, sz, i, f]
    lib.uso_gelu_fwd.restype = None
    lib.uso_gelu_bwd.argtypes = [vp, vp, vp, sz, i, f]
    lib.uso_gelu_bwd.restype = None
    lib.uso_linear_scales.argtypes = [l, l, l, i, vp, vp, vp]
    lib.uso_linear_scales.restype = None
    lib.uso_weighted_add2.argtypes = [vp, vp, vp, sz, i, f, f]
    lib.uso_weighted_add2.restype = None
    lib.uso_layer_norm_fwd.argtypes = [vp, vp, vp, vp, vp, vp, l, l, i, ctypes.c_double]
    lib.uso_layer_norm_fwd.restype = None
    lib.uso_layer_norm_bwd.argtypes = [vp, vp, vp, vp, vp, vp, l, l, i, ctypes.c_double, f]
    lib.uso_layer_norm_bwd.restype = None
    lib.uso_exponent_histogram.argtypes = [vp, i, sz, vp]
    lib.uso_exponent_histogram.restype = None
    lib.uso_cast_snr.argtypes = [vp, i, sz, i, f, vp]
    lib.uso_cast_snr.restype = None
    lib.uso_act_fwd.argtypes = [vp, vp, sz, i, i, f, f]
    lib.uso_act_fwd.restype = None
    lib.uso_act_bwd.argtypes = [vp, vp, vp, sz, i, i, f, f]
    lib.uso_act_bwd.restype = None
    _lib = lib
    return lib


_NP = {F32: np.float32, F16: np.float16, E4M3: np.uint8, E5M2: np.uint8}


def _dt_of(a: np.ndarray, dt):
    """Storage type id of an array: explicit for uint8 codes, inferred for float arrays."""
    if dt is not None:
        if a.dtype != _NP[dt]:
            raise TypeError(f"array dtype {a.dtype} does not match storage type {dt}")
        return dt
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.float16:
        return F16
    raise TypeError("FP8 code arrays (uint8) need an explicit E4M3/E5M2 type")


def _c(a: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(a)


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def cpu_threads() -> int:
    """Threads the OpenMP loops use (OMP_NUM_THREADS if set, else the visible cores)."""
    env = os.environ.get("OMP_NUM_THREADS")
    if env and env.isdigit() and int(env) > 0:
        return int(env)
    try:
        return len(os.sched_getaffinity(0))
    except AttributeError:
        return os.cpu_count() or 1


# ---- formats ---------------------------------------------------------------------------------
def decode(a: np.ndarray, dt=None) -> np.ndarray:
    """Exact value (float64) of every stored element (Sec. 3.1 value formula)."""
    a = _c(a)
    dt = _dt_of(a, dt)
    out = np.empty(a.shape, np.float64)
    _load().uso_decode(_p(a), dt, a.size, _p(out))
    return out


def encode(v: np.ndarray, dt: int, saturate: bool) -> np.ndarray:
    """Nearest representable value of each float64 (ties to even); clip or IEEE overflow."""
    v = _c(np.asarray(v, np.float64))
    out = np.empty(v.shape, _NP[dt])
    _load().uso_encode(_p(v), v.size, dt, int(saturate), _p(out))
    return out


def decode_scalar(bits: int, dt: int) -> float:
    return float(_load().uso_decode_bits(bits, dt))


def encode_scalar(v: float, dt: int, saturate: bool) -> int:
    return int(_load().uso_encode_f64(v, dt, int(saturate)))


# ---- scaled saturating cast --------------------------------------------------------------------
STAT_NAMES = ("n_sat", "n_flush0", "n_subnormal", "n_nan")


def cast_fp8(src: np.ndarray, dst_dt: int, scale: float = 1.0, src_dt=None):
    """codes = nearest-FP8(fp32(src*scale)), clipped at +-max.  Returns (codes, stats dict)."""
    src = _c(src)
    src_dt = _dt_of(src, src_dt)
    out = np.empty(src.shape, np.uint8)
    stats = np.zeros(4, np.uint64)
    _load().uso_cast_fp8(_p(src), src_dt, _p(out), dst_dt, src.size, float(np.float32(scale)), _p(stats))
    return out, {k: int(v) for k, v in zip(STAT_NAMES, stats)}


# ---- scaled matmuls ------------------------------------------------------------------------------
def linear_scales(b: int, m: int, n: int, mode: int = 0):
    """(alpha, beta_x, beta_w) as float32 (Table A.2 "Linear"; mode 1 = geometric-mean constraint)."""
    a, bx, bw = (ctypes.c_float() for _ in range(3))
    _load().uso_linear_scales(b, m, n, mode, ctypes.byref(a), ctypes.byref(bx), ctypes.byref(bw))
    return np.float32(a.value), np.float32(bx.value), np.float32(bw.value)


def _check(rc):
    if rc != 0:
        raise MemoryError("oracle could not allocate its temporaries")


def linear_fwd(X, W, alpha, x_dt=None, w_dt=None, out_dt=F16, bias=None):
    """Y[b,n] = round(alpha * X[b,m] W[m,n] (+ bias[n], an FP16 row, App. J.1's ffn))."""
    X, W = _c(X), _c(W)
    b, m = X.shape
    m2, n = W.shape
    assert m == m2
    Y = np.empty((b, n), _NP[out_dt])
    if bias is None:
        _check(_load().uso_linear_fwd(_p(X), _dt_of(X, x_dt), _p(W), _dt_of(W, w_dt), _p(Y), out_dt,
                                      b, m, n, float(np.float32(alpha))))
    else:
        bias = _c(bias)
        assert bias.dtype == np.float16 and bias.shape == (n,)
        _check(_load().uso_linear_bias_fwd(_p(X), _dt_of(X, x_dt), _p(W), _dt_of(W, w_dt), _p(bias), _p(Y), out_dt,
                                           b, m, n, float(np.float32(alpha))))
    return Y


def bias_scale(b: int):
    """beta for the gradient of a bias row summed over b rows: b^-1/2 (as layer norm's beta_c, Table A.2)."""
    return np.float32(1.0 / math.sqrt(b))


def bias_grad(G, beta_c=None, g_dt=None, out_dt=F16):
    """dc[n] = round(beta_c * sum over the b rows of G[b,n])."""
    G = _c(G)
    b, n = G.shape
    if beta_c is None:
        beta_c = bias_scale(b)
    dc = np.empty((n,), _NP[out_dt])
    _load().uso_bias_grad(_p(G), _dt_of(G, g_dt), _p(dc), out_dt, b, n, float(np.float32(beta_c)))
    return dc


def linear_bwd_dx(G, W, beta_x, g_dt=None, w_dt=None, out_dt=F16):
    """dX[b,m] = round(beta_x * G[b,n] W[m,n]^T)."""
    G, W = _c(G), _c(W)
    b, n = G.shape
    m, n2 = W.shape
    assert n == n2
    dX = np.empty((b, m), _NP[out_dt])
    _check(_load().uso_linear_bwd_dx(_p(G), _dt_of(G, g_dt), _p(W), _dt_of(W, w_dt), _p(dX), out_dt,
                                     b, m, n, float(np.float32(beta_x))))
    return dX


def linear_bwd_dw(X, G, beta_w, x_dt=None, g_dt=None, out_dt=F16):
    """dW[m,n] = round(beta_w * X[b,m]^T G[b,n])."""
    X, G = _c(X), _c(G)
    b, m = X.shape
    b2, n = G.shape
    assert b == b2
    dW = np.empty((m, n), _NP[out_dt])
    _check(_load().uso_linear_bwd_dw(_p(X), _dt_of(X, x_dt), _p(G), _dt_of(G, g_dt), _p(dW), out_dt,
                                     b, m, n, float(np.float32(beta_w))))
    return dW


# ---- unit-scaled GELU ----------------------------------------------------------------------------
def gelu_scales():
    """(alpha_g, beta_g) for gelu(x) = x*Phi(x) under z ~ N(0,1) (Table A.2 prints 1.701, 1.481).

    Rule of Sec. 5.2 "Selecting scaling factors": alpha = 1/std(gelu(z)), beta = 1/std of the
    gradient gelu'(z)*g for an independent unit-variance g, i.e. 1/rms(gelu'(z)).  Closed forms
    (Gaussian integrals):  E[gelu^2] = 1/3 + 1/(2 pi sqrt 3),  E[gelu] = 1/(2 sqrt pi),
    E[gelu'^2] = 1/3 + 2/(3 pi sqrt 3).
    """
    e2 = 1.0 / 3.0 + 1.0 / (2.0 * math.pi * math.sqrt(3.0))
    e1 = 1.0 / (2.0 * math.sqrt(math.pi))
    d2 = 1.0 / 3.0 + 2.0 / (3.0 * math.pi * math.sqrt(3.0))
    return np.float32(1.0 / math.sqrt(e2 - e1 * e1)), np.float32(1.0 / math.sqrt(d2))


def gelu_fwd(z, alpha_g):
    """h = round(alpha_g * z * Phi(z)), same storage type as z (FP16 or FP32)."""
    z = _c(z)
    dt = _dt_of(z, None)
    h = np.empty_like(z)
    _load().uso_gelu_fwd(_p(z), _p(h), z.size, dt, float(np.float32(alpha_g)))
    return h


def gelu_bwd(z, gh, beta_g):
    """gz = round(beta_g * (Phi(z) + z*phi(z)) * gh)."""
    z, gh = _c(z), _c(gh)
    dt = _dt_of(z, None)
    assert gh.dtype == z.dtype and gh.shape == z.shape
    gz = np.empty_like(z)
    _load().uso_gelu_bwd(_p(z), _p(gh), _p(gz), z.size, dt, float(np.float32(beta_g)))
    return gz


# ---- FFN chain: Linear -> unit-scaled GELU -> Linear, forward and backward -----------------------
def ffn_fwd(X16, W1_16, W2_16, fp8: bool, alpha_g=None, b1=None, b2=None):
    """Stage-by-stage forward pass with every stored intermediate kept (all roundings included).

    FP8 mode quantises only the matmul inputs (X, W1, H, W2 -> E4M3); Z, H, Y stay FP16.  b1[f], b2[d]: optional
    FP16 bias rows (App. J.1: W2 act(W1 z + b1) + b2); they are not matmul inputs and stay FP16.
    """
    if alpha_g is None:
        alpha_g = gelu_scales()[0]
    T, d = X16.shape
    f = W1_16.shape[1]
    a1 = linear_scales(T, d, f)[0]
    a2 = linear_scales(T, f, d)[0]
    r = {}
    if fp8:
        r["X8"], _ = cast_fp8(X16, E4M3)
        r["W1_8"], _ = cast_fp8(W1_16, E4M3)
        r["W2_8"], _ = cast_fp8(W2_16, E4M3)
        r["Z"] = linear_fwd(r["X8"], r["W1_8"], a1, E4M3, E4M3, bias=b1)
        r["H"] = gelu_fwd(r["Z"], alpha_g)
        r["H8"], _ = cast_fp8(r["H"], E4M3)
        r["Y"] = linear_fwd(r["H8"], r["W2_8"], a2, E4M3, E4M3, bias=b2)
    else:
        r["Z"] = linear_fwd(X16, W1_16, a1, bias=b1)
        r["H"] = gelu_fwd(r["Z"], alpha_g)
        r["Y"] = linear_fwd(r["H"], W2_16, a2, bias=b2)
    return r


def ffn_bwd(X16, W1_16, W2_16, G16, fwd: dict, fp8: bool, beta_g=None, with_bias=False):
    """Backward pass given the forward intermediates; gradients are E5M2 matmul inputs in FP8 mode.  with_bias:
    also db2 = beta * column sums of G and db1 = beta * column sums of dZ, both from the FP16 gradients (the FP8
    copies exist for the matmuls only, App. J.2)."""
    if beta_g is None:
        beta_g = gelu_scales()[1]
    T, d = X16.shape
    f = W1_16.shape[1]
    _, bx2, bw2 = linear_scales(T, f, d)   # layer 2: H[T,f] W2[f,d]
    _, bx1, bw1 = linear_scales(T, d, f)   # layer 1: X[T,d] W1[d,f]
    r = {}
    if fp8:
        r["G8"], _ = cast_fp8(G16, E5M2)
        r["dH"] = linear_bwd_dx(r["G8"], fwd["W2_8"], bx2, E5M2, E4M3)
        r["dW2"] = linear_bwd_dw(fwd["H8"], r["G8"], bw2, E4M3, E5M2)
        r["dZ"] = gelu_bwd(fwd["Z"], r["dH"], beta_g)
        r["dZ8"], _ = cast_fp8(r["dZ"], E5M2)
        r["dX"] = linear_bwd_dx(r["dZ8"], fwd["W1_8"], bx1, E5M2, E4M3)
        r["dW1"] = linear_bwd_dw(fwd["X8"], r["dZ8"], bw1, E4M3, E5M2)
    else:
        r["dH"] = linear_bwd_dx(G16, W2_16, bx2)
        r["dW2"] = linear_bwd_dw(fwd["H"], G16, bw2)
        r["dZ"] = gelu_bwd(fwd["Z"], r["dH"], beta_g)
        r["dX"] = linear_bwd_dx(r["dZ"], W1_16, bx1)
        r["dW1"] = linear_bwd_dw(X16, r["dZ"], bw1)
    if with_bias:
        r["db2"] = bias_grad(G16, bias_scale(T))
        r["db1"] = bias_grad(r["dZ"], bias_scale(T))
    return r


# ---- weighted addition and the residual FFN layer (Sec. 5.3) --------------------------------------
def weighted_add_scales(gammas):
    """Table A.2 "weighted_add": sum_i gamma_i x_i has alpha = (sum gamma_i^2)^-1/2, beta_i = 1/gamma_i."""
    g = [float(x) for x in gammas]
    return 1.0 / math.sqrt(sum(x * x for x in g)), [1.0 / x for x in g]


def residual_weights(tau: float):
    """fixed(tau) interpolation of Sec. 5.3: (skip, branch) = (sqrt(1-tau), sqrt(tau)), as the floats the library uses.
    The branch weight is rounded to float first and the skip weight derived from it, sqrt(1 - branch^2), the way the
    library derives it from the one scale it is given."""
    branch = np.float32(math.sqrt(tau))
    skip = np.float32(math.sqrt(1.0 - float(branch) * float(branch)))
    return skip, branch


def weighted_add2(a, b, ca, cb):
    """round(ca*a + cb*b) in the storage type of a and b."""
    a, b = _c(a), _c(b)
    dt = _dt_of(a, None)
    assert a.dtype == b.dtype and a.shape == b.shape
    out = np.empty_like(a)
    _load().uso_weighted_add2(_p(a), _p(b), _p(out), a.size, dt, float(np.float32(ca)), float(np.float32(cb)))
    return out


def ffn_res_fwd(X16, W1_16, W2_16, tau: float, fp8: bool):
    """Residual FFN layer (Fig. 3, right): out = sqrt(1-tau) x + sqrt(tau) FFN(x).  r["Y"] is the branch output
    FFN(x) as stored FP16, r["Out"] the layer output."""
    r = ffn_fwd(X16, W1_16, W2_16, fp8)
    skip, branch = residual_weights(tau)
    r["Out"] = weighted_add2(X16, r["Y"], skip, branch)
    return r


def ffn_res_bwd(X16, W1_16, W2_16, G16, fwd: dict, tau: float, fp8: bool):
    """Backward of the residual layer: the branch receives the incoming gradient unscaled (so dW1, dW2 and dZ are
    those of the plain FFN), and grad_x = sqrt(1-tau) g + sqrt(tau) grad_x_branch."""
    r = ffn_bwd(X16, W1_16, W2_16, G16, fwd, fp8)
    skip, branch = residual_weights(tau)
    r["dXin"] = weighted_add2(G16, r["dX"], skip, branch)
    return r


# ---- the other activations of Table A.2 ------------------------------------------------------------
GELU, RELU, TANH, SIGMOID = 0, 1, 2, 3


def act_scales(kind: int):
    """(alpha, beta) of an activation under z ~ N(0,1), by the rule of Sec. 5.2: alpha = 1/std(f(z)),
    beta = 1/rms(f'(z)).  relu has closed forms (App. E.1): Var = (1 - 1/pi)/2 and E[f'^2] = 1/2; gelu: gelu_scales();
    tanh and sigmoid by Gauss-Hermite quadrature (the paper found them "empirically": 1.593/1.467 and 4.802/4.722)."""
    if kind == GELU:
        return gelu_scales()
    if kind == RELU:
        return np.float32(math.sqrt(2.0 / (1.0 - 1.0 / math.pi))), np.float32(math.sqrt(2.0))
    x, w = np.polynomial.hermite_e.hermegauss(200)
    w = w / math.sqrt(2.0 * math.pi)
    if kind == TANH:
        f, df = np.tanh(x), 1.0 / np.cosh(x) ** 2
    elif kind == SIGMOID:
        sg = 1.0 / (1.0 + np.exp(-x))
        f, df = sg, sg * (1.0 - sg)
    else:
        raise ValueError(kind)
    mean = float(np.sum(w * f))
    var = float(np.sum(w * f * f)) - mean * mean
    return np.float32(1.0 / math.sqrt(var)), np.float32(1.0 / math.sqrt(float(np.sum(w * df * df))))


def act_fwd(z, kind: int, scale, s1=1.0):
    """h = round(scale * f(s1 * z)), storage type of z."""
    z = _c(z)
    h = np.empty_like(z)
    _load().uso_act_fwd(_p(z), _p(h), z.size, _dt_of(z, None), kind, float(np.float32(s1)), float(np.float32(scale)))
    return h


def act_bwd(z, gh, kind: int, scale, s1=1.0):
    """gz = round(scale * f'(s1 * z) * gh)."""
    z, gh = _c(z), _c(gh)
    assert gh.dtype == z.dtype and gh.shape == z.shape
    gz = np.empty_like(z)
    _load().uso_act_bwd(_p(z), _p(gh), _p(gz), z.size, _dt_of(z, None), kind, float(np.float32(s1)), float(np.float32(scale)))
    return gz


# ---- scaled layer norm (Table A.2 "Other") -----------------------------------------------------------
def layer_norm_scales(b: int):
    """alpha = 1, beta_x = 1, beta_w = beta_c = b^-1/2 (b = rows, i.e. tokens)."""
    return 1.0, 1.0, np.float32(1.0 / math.sqrt(b))


def layer_norm_fwd(X, w, c, eps: float = 0.0):
    """Returns (Y, mean, rstd): Y in the storage type of X, the row statistics in float64."""
    X, w, c = _c(X), _c(w), _c(c)
    b, n = X.shape
    assert w.shape == (n,) and c.shape == (n,) and w.dtype == X.dtype and c.dtype == X.dtype
    Y = np.empty_like(X)
    mean, rstd = np.empty(b, np.float64), np.empty(b, np.float64)
    _load().uso_layer_norm_fwd(_p(X), _p(w), _p(c), _p(Y), _p(mean), _p(rstd), b, n, _dt_of(X, None), float(eps))
    return Y, mean, rstd


def layer_norm_bwd(X, w, G, eps: float = 0.0, beta_wc=None):
    """Returns (dX, dw, dc) for the incoming gradient G[b,n]."""
    X, w, G = _c(X), _c(w), _c(G)
    b, n = X.shape
    assert G.shape == X.shape and G.dtype == X.dtype and w.shape == (n,)
    if beta_wc is None:
        beta_wc = layer_norm_scales(b)[2]
    dX, dw, dc = np.empty_like(X), np.empty_like(w), np.empty_like(w)
    _load().uso_layer_norm_bwd(_p(X), _p(w), _p(G), _p(dX), _p(dw), _p(dc), b, n, _dt_of(X, None), float(eps),
                               float(np.float32(beta_wc)))
    return dX, dw, dc


# ---- diagnostics: exponent histogram (Fig. 1, App. K) and SNR of a cast (Sec. 3.1) ---------------------
HIST_BINS = 35


def exponent_histogram(a: np.ndarray) -> np.ndarray:
    """Counts per bin: 0 zero, 1 below 2^-24, 2 [2^-24, 2^-14), 3 + (e + 14) for exponent e = -14..15, 33 >= 2^16 / inf, 34 NaN."""
    a = _c(a)
    hist = np.zeros(HIST_BINS, np.uint64)
    _load().uso_exponent_histogram(_p(a), _dt_of(a, None), a.size, _p(hist))
    return hist


def cast_snr(a: np.ndarray, dst_dt: int, scale: float = 1.0):
    """(sum x^2, sum (q(x*scale)/scale - x)^2); their ratio is the SNR of Sec. 3.1."""
    a = _c(a)
    sums = np.zeros(2, np.float64)
    _load().uso_cast_snr(_p(a), _dt_of(a, None), a.size, dst_dt, float(np.float32(scale)), _p(sums))
    return float(sums[0]), float(sums[1])


# ---- scaled sum over the last dimension (Table A.2 "Linear") -------------------------------------------------------
def sum_scales(n: int):
    """(alpha, beta) = (n^-1/2, 1)."""
    return np.float32(1.0 / math.sqrt(n)), np.float32(1.0)


def sum_fwd(x, alpha=None):
    """y[rows] = round(alpha * sum over the last dimension of FP16 x[rows, n])."""
    x = _c(x)
    assert x.dtype == np.float16 and x.ndim == 2
    rows, n = x.shape
    if alpha is None:
        alpha = sum_scales(n)[0]
    y = np.empty(rows, np.float16)
    _load().uso_sum_fwd(_p(x), _p(y), rows, n, float(np.float32(alpha)))
    return y


def sum_bwd(g, n: int, beta=1.0):
    """dx[rows, n] = round(beta * g[rows]) in every column."""
    g = _c(g)
    assert g.dtype == np.float16 and g.ndim == 1
    dx = np.empty((g.shape[0], n), np.float16)
    _load().uso_sum_bwd(_p(g), _p(dx), g.shape[0], n, float(np.float32(beta)))
    return dx


# ---- scaled softmax and softmax cross-entropy (Table A.2 "Other", App. G) ---------------------------------
def softmax_scales(s: int):
    """(alpha, beta) = (s, s): the output of a softmax over s unit-normal values is about 1/s everywhere, so s times
    it is about a vector of ones for the matmul that follows (App. G "Softmax (followed by matmul)")."""
    return np.float32(s), np.float32(s)


def softmax_xent_scale(s: int):
    """beta = s / sqrt(s - 1) (App. G "Softmax cross-entropy"; alpha = 1)."""
    return np.float32(s / math.sqrt(s - 1.0))


def softmax_fwd(x, alpha=None, s1=1.0):
    """y = round(alpha * softmax(s1 * x)) over the last dimension of an FP16 [rows, s] array."""
    x = _c(x)
    assert x.dtype == np.float16 and x.ndim == 2
    rows, s = x.shape
    if alpha is None:
        alpha = softmax_scales(s)[0]
    y = np.empty_like(x)
    _load().uso_softmax_fwd(_p(x), _p(y), rows, s, float(np.float32(s1)), float(np.float32(alpha)))
    return y


def softmax_bwd(x, g, beta=None, s1=1.0):
    """dx = round(beta * s1 * p * (g - sum(p * g))), p = softmax(s1 * x)."""
    x, g = _c(x), _c(g)
    assert x.dtype == np.float16 and g.dtype == np.float16 and x.shape == g.shape and x.ndim == 2
    rows, s = x.shape
    if beta is None:
        beta = softmax_scales(s)[1]
    dx = np.empty_like(x)
    _load().uso_softmax_bwd(_p(x), _p(g), _p(dx), rows, s, float(np.float32(s1)), float(np.float32(beta)))
    return dx


def softmax_xent(x, target, beta=None, s1=1.0):
    """(loss[rows] float64, dx[rows, s] FP16): loss = -log softmax(s1 x)_target, dx = round(beta * s1 * (p - onehot));
    rows whose target lies outside 0 .. s-1 carry no label: loss 0, gradient 0."""
    x = _c(x)
    target = np.ascontiguousarray(target, dtype=np.int32)
    assert x.dtype == np.float16 and x.ndim == 2 and target.shape == (x.shape[0],)
    rows, s = x.shape
    if beta is None:
        beta = softmax_xent_scale(s)
    loss = np.empty(rows, np.float64)
    dx = np.empty_like(x)
    _load().uso_softmax_xent(_p(x), _p(target), _p(loss), _p(dx), rows, s, float(np.float32(s1)), float(np.float32(beta)))
    return loss, dx


# ---- batched scaled matmuls and unit-scaled dot-product attention (App. F "Scaled dot product self attention",
#      Table A.2 "Linear" for the factors of each product, App. G for the softmax between them) -------------------
def matmul_batched(A, B, scale, trans_a=False, trans_b=False, a_dt=None, b_dt=None, out_dt=F16):
    """C[i] = round(scale * op(A[i]) op(B[i])) for every i of the leading (batch) dimension; op transposes the last
    two dimensions where asked.  Each slice is the plain matmul of this module (double sums in index order)."""
    assert not (trans_a and trans_b)
    outs = []
    for a, b in zip(A, B):
        if not trans_a and not trans_b:
            outs.append(linear_fwd(a, b, scale, a_dt, b_dt, out_dt))            # [M,K] [K,N]
        elif trans_b:
            outs.append(linear_bwd_dx(a, b, scale, a_dt, b_dt, out_dt))         # [M,K] [N,K]^T
        else:
            outs.append(linear_bwd_dw(a, b, scale, a_dt, b_dt, out_dt))         # [K,M]^T [K,N]
    return np.stack(outs)


def attention_scales(s: int, d: int):
    """Factors of the three ops of one attention head with s keys and head size d, by Table A.2's matmul rule
    (alpha = fan_in^-1/2, beta_X = fan_out^-1/2, beta_W = rows^-1/2) and its softmax row:
      scores  A = Q K^T : reduces over d, its two gradients over s;  probabilities: alpha = beta = s;
      output  O = P V   : reduces over s, grad_P over d, grad_V over the s queries."""
    r = lambda v: np.float32(1.0 / math.sqrt(v))
    return dict(a_scores=r(d), b_q=r(s), b_k=r(s), a_soft=np.float32(s), b_soft=np.float32(s), a_out=r(s), b_p=r(d), b_v=r(s))


def attention_fwd(Q, K, V):
    """Unit-scaled dot-product attention for FP16 Q, K, V of shape [heads, s, d] (no mask): every stored tensor kept."""
    h, s, d = Q.shape
    c = attention_scales(s, d)
    r = {}
    r["A"] = matmul_batched(Q, K, c["a_scores"], trans_b=True)                   # [h, s, s]
    r["P"] = softmax_fwd(r["A"].reshape(h * s, s), c["a_soft"]).reshape(h, s, s)
    r["O"] = matmul_batched(r["P"], V, c["a_out"])                               # [h, s, d]
    return r


def attention_bwd(Q, K, V, dO, fwd: dict):
    """Backward of attention_fwd from its stored A and P."""
    h, s, d = Q.shape
    c = attention_scales(s, d)
    r = {}
    r["dV"] = matmul_batched(fwd["P"], dO, c["b_v"], trans_a=True)               # P^T dO   [h, s, d]
    r["dP"] = matmul_batched(dO, V, c["b_p"], trans_b=True)                      # dO V^T   [h, s, s]
    r["dA"] = softmax_bwd(fwd["A"].reshape(h * s, s), r["dP"].reshape(h * s, s), c["b_soft"]).reshape(h, s, s)
    r["dQ"] = matmul_batched(r["dA"], K, c["b_q"])                               # dA K     [h, s, d]
    r["dK"] = matmul_batched(r["dA"], Q, c["b_k"], trans_a=True)                 # dA^T Q   [h, s, d]
    return r
