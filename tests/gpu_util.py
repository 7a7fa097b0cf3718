"""Helpers for the GPU parity tests: numpy <-> device buffers through PyTorch (memory and streams
only), calls into the HIP library through its ctypes binding, and the GEMM error metric."""
from __future__ import annotations

import numpy as np
import torch

import paper_2303_11257_amd as us
import parity

DEV = "cuda:0"
_TORCH = {np.dtype(np.float16): torch.float16, np.dtype(np.float32): torch.float32, np.dtype(np.uint8): torch.uint8}


def to_dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def empty(shape, dtype) -> torch.Tensor:
    return torch.empty(shape, dtype=_TORCH[np.dtype(dtype)], device=DEV)


def to_np(t: torch.Tensor) -> np.ndarray:
    torch.cuda.synchronize()
    return t.cpu().numpy()


def stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def ptr(t):
    return None if t is None else t.data_ptr()


def np_dt(a) -> int:
    return {np.dtype(np.float16): us.F16, np.dtype(np.float32): us.F32}[np.dtype(a.dtype)]


# ---- thin wrappers: numpy in, numpy out, every step on the GPU -----------------------------------
def cast_fp8(x: np.ndarray, dst_dt: int, scale: float = 1.0, want_stats: bool = False):
    src = to_dev(x.reshape(-1))
    dst = empty((x.size,), np.uint8)
    stats = torch.zeros(4, dtype=torch.int64, device=DEV) if want_stats else None
    us.cast_fp8(ptr(src), np_dt(x), ptr(dst), dst_dt, x.size, scale, ptr(stats), stream())
    codes = to_np(dst).reshape(x.shape)
    if want_stats:
        s = to_np(stats)
        return codes, dict(n_sat=int(s[0]), n_flush0=int(s[1]), n_subnormal=int(s[2]), n_nan=int(s[3]))
    return codes


def linear_fwd(X, W, x_dt, w_dt, alpha=0.0, out_dt=us.F16, epi=us.EPI_NONE, epi_scale=0.0, want16=True, want8=False,
               workspace_bytes=0, skip=None):
    b, m = X.shape
    n = W.shape[1]
    dX_, dW_ = to_dev(X), to_dev(W)
    Y = empty((b, n), np.float16 if out_dt == us.F16 else np.float32)
    base = epi & 0xf                                # without the activation-kind and table flags
    a16 = empty((b, n), np.float16) if (base == us.EPI_GELU and want16) else None
    if base == us.EPI_RESIDUAL:
        a16 = to_dev(skip)                          # an input here: the skip tensor of the interpolation
    a8 = empty((b, n), np.uint8) if (base == us.EPI_GELU and want8) else None
    ws = torch.empty(workspace_bytes, dtype=torch.uint8, device=DEV) if workspace_bytes else None
    us.linear_fwd(ptr(dX_), ptr(dW_), ptr(Y), b, m, n, x_dt, w_dt, out_dt, alpha, epi, epi_scale, ptr(a16), ptr(a8),
                  ptr(ws), workspace_bytes, stream())
    out = [to_np(Y)]
    if base == us.EPI_GELU:
        out += [to_np(a16) if a16 is not None else None, to_np(a8) if a8 is not None else None]
    return out[0] if len(out) == 1 else tuple(out)


def linear_bwd(X, W, G, x_dt, w_dt, g_dt, beta_x=0.0, beta_w=0.0, out_dt=us.F16, epi=us.EPI_NONE, epi_scale=0.0,
               Zpre=None, want8=False, do_dx=True, do_dw=True, no_workspace=False, store_dx=True):
    b, n = G.shape
    m = W.shape[0] if W is not None else X.shape[1]
    tX = to_dev(X) if X is not None else None
    tW = to_dev(W) if W is not None else None
    tG = to_dev(G)
    odt = np.float16 if out_dt == us.F16 else np.float32
    dX = empty((b, m), odt) if (do_dx and store_dx) else None      # store_dx=False: GELU' epilogue, codes only
    dW = empty((m, n), odt) if do_dw else None
    tZ = to_dev(Zpre) if Zpre is not None else None
    a8 = empty((b, m), np.uint8) if want8 else None
    wsb = 0 if no_workspace else us.workspace_bytes(b, m, n)
    ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device=DEV)
    us.linear_bwd(ptr(tX), ptr(tW), ptr(tG), ptr(dX), ptr(dW), b, m, n, x_dt, w_dt, g_dt, out_dt, beta_x, beta_w, epi,
                  epi_scale, ptr(tZ), ptr(a8), ptr(ws), wsb, stream())
    return (to_np(dX) if dX is not None else None, to_np(dW) if do_dw else None, to_np(a8) if want8 else None)


# ---- error metric for matmul / GELU outputs (tests/parity.py) ------------------------------------------
TAU = parity.TAU
RTOL = parity.RTOL
_record = None        # the running test's record_property (set by conftest.py), so every comparison leaves its figures


def rel_err(gpu: np.ndarray, ref: np.ndarray, fp8: bool = False, scale: float = 1.0) -> float:
    return parity.errors(gpu, ref, fp8, scale)["gated"]


def assert_close(gpu, ref, what="", fp8=False, scale=1.0, tau=parity.TAU, allow=None):
    """fp8: the compared value comes out of a product of FP8 operands (absolute floor of the matrix core's adder)."""
    e = parity.errors(gpu, ref, fp8, scale, tau, allow)
    if _record is not None:
        for k in ("gated", "unfloored_max", "rms"):
            _record(f"{what or 'tensor'}:{k}", e[k])
    print(f"parity {what}: gated {e['gated']:.2e}  un-floored max {e['unfloored_max']:.2e}  rms {e['rms']:.2e}")
    assert e["gated"] <= RTOL, f"{what}: max relative error {e['gated']:.3e} > {RTOL} (un-floored {e['unfloored_max']:.3e}, rms {e['rms']:.3e})"
    return e["gated"]
