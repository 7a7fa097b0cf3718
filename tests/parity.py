"""The error metric of the GPU parity tests, in one place (plain numpy; the smoke check uses it too).

    gated = max_i  max(|gpu_i - ref_i| - A*S, 0) / max(|ref_i|, tau*S)   <=  2e-3

ref is the oracle on the same stored operands.  S is the scale of the tensor (1 for the unit-scaled tensors of the
method; the range-stress products pass the RMS of their reference).  tau = 2^-6: below 1.6 % of one standard deviation
the bound turns absolute (2e-3 * 2^-6 = 3.1e-5, two FP16 steps at that magnitude; FP32 accumulation over K = 16384
unit-scale products contributes about 4e-6 there).  A is zero for FP16 operands, GELU, the activations and the residual
add.  For FP8 operands A = 2e-4: the matrix core adds the products of a group in a narrow adder, which leaves an absolute
error that does not shrink with |ref| (measured on unit-scale outputs for K = 64 ... 8192: at most 9e-5, RMS 1.4e-5).
Besides the gated figure every comparison reports the un-floored maximum relative error (over ref != 0) and the RMS error.
"""
from __future__ import annotations

import numpy as np

RTOL = 2e-3
TAU = 2.0 ** -6
FP8_ABS = 2e-4


def errors(gpu: np.ndarray, ref: np.ndarray, fp8: bool = False, scale: float = 1.0, tau: float = TAU, allow=None) -> dict:
    """allow: optional per-element absolute allowance added to A*S (the range-stress products pass 2^-12 * sum_k |x_k w_k|)."""
    g, r = np.asarray(gpu).astype(np.float64), np.asarray(ref).astype(np.float64)
    same_inf = np.isinf(g) & np.isinf(r) & (np.sign(g) == np.sign(r))
    both_nan = np.isnan(g) & np.isnan(r)
    agree = same_inf | both_nan                                # compared by class: no error
    with np.errstate(invalid="ignore"):
        d = np.where(agree, 0.0, np.abs(g - r))
    d = np.where(np.isnan(d), np.inf, d)                       # NaN or inf on one side only, or inf of opposite signs
    a = FP8_ABS * scale if fp8 else 0.0
    if allow is not None:
        a = a + np.asarray(allow, np.float64)
    den = np.where(np.isfinite(r), np.maximum(np.abs(r), tau * scale), 1.0)
    excess = np.where(np.isinf(d), np.inf, np.maximum(d - a, 0.0))
    gated = float(np.max(excess / den)) if d.size else 0.0
    nz = (r != 0) & np.isfinite(r)
    unfloored = float(np.max(d[nz] / np.abs(r[nz]))) if nz.any() else 0.0
    fin = np.isfinite(d)
    rms = float(np.sqrt(np.mean(d[fin] ** 2))) if fin.any() else 0.0
    return dict(gated=gated, unfloored_max=unfloored, rms=rms, max_abs=float(d.max()) if d.size else 0.0)
