"""Seeded synthetic inputs for the unit-scaled linear / FFN tests and benchmarks.

This module serves both the CPU oracle's tests and the GPU path's tests; it holds none of the
method's arithmetic (no scaling rules, no FP8 rounding, no matmul, no GELU).  It only draws
numbers: a counter-based generator, so element ``i`` of tensor ``t`` under seed ``s`` is a pure
function of ``(s, t, i)`` and any slice can be produced independently of the rest.

The paper trains on text corpora; at initialisation every tensor of a unit-scaled model is close
to N(0,1) (Sec. 4 "ideal scaling criterion", Sec. 5.2), which is what these draws stand in for.
Shapes follow Table A.5 (hidden 768/1024, FFN 3072/4096, sequence 128).
"""
from __future__ import annotations

import numpy as np

# tensor ids
T_X, T_W1, T_W2, T_G = 1, 2, 3, 4
BASE_SEED = 20230311

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


def _mix(x: np.ndarray) -> np.ndarray:
    """64-bit avalanche mixer (the splitmix64 finaliser)."""
    x = x.astype(np.uint64, copy=True)
    with np.errstate(over="ignore"):
        x ^= x >> np.uint64(30)
        x *= np.uint64(0xBF58476D1CE4E5B9)
        x ^= x >> np.uint64(27)
        x *= np.uint64(0x94D049BB133111EB)
        x ^= x >> np.uint64(31)
    return x


def _stream(seed: int, tensor: int, lane: int, start: int, count: int) -> np.ndarray:
    """``count`` 64-bit words for counters start..start+count-1 of stream (seed, tensor, lane)."""
    with np.errstate(over="ignore"):
        key = _mix(np.array([(seed * 0x9E3779B97F4A7C15 + tensor * 0xD1B54A32D192ED03 + lane * 0x8CB92BA72F3D8DD7)
                             & 0xFFFFFFFFFFFFFFFF], dtype=np.uint64))[0]
        ctr = np.arange(start, start + count, dtype=np.uint64)
        return _mix(ctr * np.uint64(0x9E3779B97F4A7C15) + key)


def uniform01(seed: int, tensor: int, lane: int, start: int, count: int) -> np.ndarray:
    """float64 uniforms in (0,1): (top 53 bits + 0.5) / 2^53."""
    w = _stream(seed, tensor, lane, start, count)
    return ((w >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def normal(seed: int, tensor: int, shape, sigma: float = 1.0, dtype=np.float16, start: int = 0) -> np.ndarray:
    """i.i.d. N(0, sigma^2): Box-Muller in float64, rounded once to float32, then to ``dtype``."""
    count = int(np.prod(shape))
    out = np.empty(count, dtype=dtype)
    chunk = 1 << 22
    for lo in range(0, count, chunk):
        n = min(chunk, count - lo)
        u1 = uniform01(seed, tensor, 0, start + lo, n)
        u2 = uniform01(seed, tensor, 1, start + lo, n)
        z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
        out[lo:lo + n] = (z * sigma).astype(np.float32).astype(dtype)
    return out.reshape(shape)


def outlier_positions(seed: int, tensor: int, count: int, one_in: int = 1000):
    """Which of ``count`` elements are outliers, and their signs: element i is one iff word(i) % one_in == 0; its sign
    is the word's top bit.  Returns (indices, signs as +-1.0 float32)."""
    idx, sgn = [], []
    chunk = 1 << 22
    for lo in range(0, count, chunk):
        n = min(chunk, count - lo)
        w = _stream(seed, tensor, 2, lo, n)
        hit = np.nonzero((w % np.uint64(one_in)) == 0)[0]
        idx.append(hit + lo)
        sgn.append(np.where((w[hit] >> np.uint64(63)) == 1, -1.0, 1.0).astype(np.float32))
    return np.concatenate(idx), np.concatenate(sgn)


def place_outliers(base: np.ndarray, sigma: float, positions, outlier: float = 1000.0) -> np.ndarray:
    """``base`` (FP32 draws of N(0,1)) scaled by ``sigma`` with +-outlier written at ``positions`` (from
    outlier_positions): for a sigma that is a power of two this is normal_with_outliers(seed, tensor, shape, sigma)
    without drawing the normals again (the scaling is exact)."""
    a = (base.astype(np.float32) * np.float32(sigma)).reshape(-1)
    idx, sgn = positions
    a[idx] = sgn * np.float32(outlier)
    return a.reshape(base.shape)


def normal_with_outliers(seed: int, tensor: int, shape, sigma: float, outlier: float = 1000.0,
                         one_in: int = 1000, dtype=np.float32):
    """N(0, sigma^2) with one element in ``one_in`` replaced by +-outlier (range-stress inputs).

    Returns (array, number of outliers).  Element i is an outlier iff word(i) % one_in == 0; its
    sign is the word's top bit.
    """
    a = normal(seed, tensor, shape, sigma, np.float32).reshape(-1)
    idx, sgn = outlier_positions(seed, tensor, a.size, one_in)
    a[idx] = sgn * np.float32(outlier)
    return a.astype(dtype).reshape(shape), int(idx.size)


def small_ints(seed: int, tensor: int, shape, lo: int = -2, hi: int = 2, dtype=np.float16) -> np.ndarray:
    """Uniform integers in [lo, hi] (exactly representable in FP16 / E4M3 / E5M2 for |v| <= 2)."""
    count = int(np.prod(shape))
    w = _stream(seed, tensor, 3, 0, count)
    v = (w % np.uint64(hi - lo + 1)).astype(np.int64) + lo
    return v.astype(dtype).reshape(shape)


# ---- the workloads named by the benchmark configuration ---------------------------------------
CONFIGS = {
    # name: (kind, tokens, d_model, d_ff, fp8)
    "C1": dict(kind="linear", b=256, m=256, n=1024, fp8=False, seed=BASE_SEED + 0),
    "C2": dict(kind="ffn", T=4096, d=768, f=3072, fp8=False, seed=BASE_SEED + 1),
    "C3": dict(kind="ffn", T=8192, d=1024, f=4096, fp8=True, seed=BASE_SEED + 2),
    "C5": dict(kind="ffn", T=32768, d=4096, f=16384, fp8=True, seed=BASE_SEED + 4),
}
C4_SIZES = (2048, 4096, 8192)
C4_SIGMAS = (1.0 / 64, 1.0 / 8, 1.0, 8.0, 64.0)
C4_SEED = BASE_SEED + 3


def linear_inputs(b: int, m: int, n: int, seed: int):
    """X[b,m], W[m,n], G[b,n], all FP16 N(0,1)."""
    return (normal(seed, T_X, (b, m)), normal(seed, T_W1, (m, n)), normal(seed, T_G, (b, n)))


def ffn_inputs(T: int, d: int, f: int, seed: int):
    """X[T,d], W1[d,f], W2[f,d], G[T,d], all FP16 N(0,1) (unit-scaled initialisation)."""
    return (normal(seed, T_X, (T, d)), normal(seed, T_W1, (d, f)), normal(seed, T_W2, (f, d)),
            normal(seed, T_G, (T, d)))


def normal_on_device(seed: int, tensor: int, shape, device="cuda:0"):
    """FP16 N(0,1) drawn on the GPU by PyTorch's seeded Philox generator.

    For the largest workload only (hundreds of millions of elements), where the numpy generator above
    would take minutes; slabs of the result are copied back for the oracle.  Returns a torch tensor.
    """
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(seed * 1000003 + tensor)
    return torch.randn(shape, generator=g, device=device, dtype=torch.float32).to(torch.float16)
