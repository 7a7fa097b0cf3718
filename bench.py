#!/usr/bin/env python3
"""Benchmark of the unit-scaled FFN forward + backward on one MI355X.

One step = one pass of the whole hot path over one batch that is already resident in HBM:
FP8 casts of X, W1, W2 (E4M3) and G (E5M2), Linear+GELU, Linear, and the four backward products
(grad_X with GELU' fused, grad_W twice).  The headline workload is the FP8 BERT-large FFN
(tokens 8192 = 64 x 128, d_model 1024, d_ff 4096); the FP16 BERT-base FFN and the cast kernel's
bandwidth are reported beside it.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C3|C2|C5] [--no-cpu-baseline] [--no-secondary]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"fp8": 5000.0, "f16": 2500.0}   # dense MFMA peaks of MI355X
PEAK_HBM_GBS = 8000.0

WORKLOADS = {
    "C2": dict(T=4096, d=768, f=3072, fp8=False, desc="unit-scaled FFN fwd+bwd, FP16, BERT-base shape"),
    "C3": dict(T=8192, d=1024, f=4096, fp8=True, desc="unit-scaled FFN fwd+bwd, FP8 (E4M3 fwd / E5M2 grads), BERT-large shape"),
    "C5": dict(T=32768, d=4096, f=16384, fp8=True, desc="unit-scaled FFN fwd+bwd, FP8, LLM-size shape"),
}


class Ffn:
    """Device buffers for one workload and the calls of one step."""

    def __init__(self, torch, us, synth, T, d, f, fp8, seed):
        self.torch, self.us = torch, us
        self.T, self.d, self.f, self.fp8 = T, d, f, fp8
        dev = "cuda:0"
        self.X = synth.normal_on_device(seed, synth.T_X, (T, d), dev)
        self.W1 = synth.normal_on_device(seed, synth.T_W1, (d, f), dev)
        self.W2 = synth.normal_on_device(seed, synth.T_W2, (f, d), dev)
        self.G = synth.normal_on_device(seed, synth.T_G, (T, d), dev)
        e = lambda shape, dt=torch.float16: torch.empty(shape, dtype=dt, device=dev)
        u8 = torch.uint8
        if fp8:
            self.X8, self.W1_8, self.W2_8, self.G8 = e((T, d), u8), e((d, f), u8), e((f, d), u8), e((T, d), u8)
        self.Z, self.Y = e((T, f)), e((T, d))
        self.H = e((T, f), u8 if fp8 else torch.float16)
        self.dX, self.dW1, self.dW2 = e((T, d)), e((d, f)), e((f, d))
        # grad of the pre-activation: FP16 in the FP16 step; in the FP8 step only its E5M2 codes are stored
        # (they are all the layer-1 backward matmuls read)
        self.dZ16 = None if fp8 else e((T, f))
        self.dZ8 = e((T, f), u8) if fp8 else None
        self.wsb = max(us.ffn_workspace_bytes(T, d, f), us.ffn_bias_workspace_bytes(T, d, f))
        self.ws = torch.empty(max(self.wsb, 16), dtype=u8, device=dev)
        # the GELU tables depend on the two scale factors only: built once here, like the workspace itself
        us.gelu_tables(self.ws.data_ptr(), self.wsb, 0.0, 0.0, torch.cuda.current_stream().cuda_stream)
        self.mode = (us.FFN_FP8 if fp8 else 0) | us.FFN_TABLES_READY
        self.flop = 12.0 * T * d * f

    def p(self, t):
        return None if t is None else t.data_ptr()

    def calls(self):
        """The launches of the step, one by one, as (name, kind, flop, bytes, thunk): the same calls, in the same
        order, that us_ffn_fwd / us_ffn_bwd make."""
        us, p, st = self.us, self.p, self.torch.cuda.current_stream().cuda_stream
        T, d, f = self.T, self.d, self.f
        gemm = 2.0 * T * d * f
        out = []
        if self.fp8:
            op, gr = us.E4M3, us.E5M2
            X, W1, W2, G = self.X8, self.W1_8, self.W2_8, self.G8
            srcs, dsts = [self.X, self.W1, self.W2, self.G], [X, W1, W2, G]
            ns = [t.numel() for t in srcs]
            out.append(("cast_batch", "cast", 0.0, 3.0 * sum(ns),
                        lambda: us.cast_fp8_batch([p(t) for t in srcs], [p(t) for t in dsts], ns, [op, op, op, gr], st)))
        else:
            op = gr = us.F16
            X, W1, W2, G = self.X, self.W1, self.W2, self.G
        a16, a8 = (None, self.H) if self.fp8 else (self.H, None)
        out.append(("fwd1_gelu", "gemm", gemm, 0.0, lambda: us.linear_fwd(p(X), p(W1), p(self.Z), T, d, f, op, op, us.F16, 0.0,
                                                                         us.EPI_GELU | us.EPI_TABLES_READY, 0.0, p(a16), p(a8), p(self.ws), self.wsb, st)))
        out.append(("fwd2", "gemm", gemm, 0.0, lambda: us.linear_fwd(p(self.H), p(W2), p(self.Y), T, f, d, op, op, us.F16, 0.0,
                                                                    us.EPI_NONE, 0.0, None, None, None, 0, st)))
        # backward: one call per layer computes grad_X and grad_W (one launch where the shapes allow it)
        out.append(("bwd2_dx_gelugrad_dw", "gemm", 2 * gemm, 0.0,
                    lambda: us.linear_bwd(p(self.H), p(W2), p(G), p(self.dZ16), p(self.dW2), T, f, d, op, op, gr, us.F16, 0.0, 0.0,
                                          us.EPI_GELU_GRAD | us.EPI_TABLES_READY, 0.0, p(self.Z), p(self.dZ8), p(self.ws), self.wsb, st)))
        dZ = self.dZ8 if self.fp8 else self.dZ16
        out.append(("bwd1_dx_dw", "gemm", 2 * gemm, 0.0,
                    lambda: us.linear_bwd(p(X), p(W1), p(dZ), p(self.dX), p(self.dW1), T, d, f, op, op, gr, us.F16, 0.0, 0.0,
                                          us.EPI_NONE, 0.0, None, None, p(self.ws), self.wsb, st)))
        return out

    def step(self):
        """The step through the two FFN entry points (what `value` times)."""
        us, p, st = self.us, self.p, self.torch.cuda.current_stream().cuda_stream
        T, d, f = self.T, self.d, self.f
        if self.fp8:
            us.cast_fp8_batch([p(self.X), p(self.W1), p(self.W2), p(self.G)], [p(self.X8), p(self.W1_8), p(self.W2_8), p(self.G8)],
                              [self.X.numel(), self.W1.numel(), self.W2.numel(), self.G.numel()],
                              [us.E4M3, us.E4M3, us.E4M3, us.E5M2], st)
            X, W1, W2, G = self.X8, self.W1_8, self.W2_8, self.G8
        else:
            X, W1, W2, G = self.X, self.W1, self.W2, self.G
        us.ffn_fwd(p(X), p(W1), p(W2), p(self.Z), p(self.H), p(self.Y), T, d, f, self.mode, p(self.ws), self.wsb, st)
        us.ffn_bwd(p(X), p(W1), p(W2), p(self.Z), p(self.H), p(G), p(self.dZ16), p(self.dZ8), p(self.dX), p(self.dW1),
                   p(self.dW2), T, d, f, self.mode, p(self.ws), self.wsb, st)

    def step_act_casts_only(self):
        """The step of a training loop with gradient accumulation (App. J.2: the weights change once per many
        micro-batches): only the activation X and the gradient G are cast, the E4M3 weights are reused."""
        us, p, st = self.us, self.p, self.torch.cuda.current_stream().cuda_stream
        T, d, f = self.T, self.d, self.f
        us.cast_fp8_batch([p(self.X), p(self.G)], [p(self.X8), p(self.G8)], [self.X.numel(), self.G.numel()], [us.E4M3, us.E5M2], st)
        us.ffn_fwd(p(self.X8), p(self.W1_8), p(self.W2_8), p(self.Z), p(self.H), p(self.Y), T, d, f, self.mode, p(self.ws), self.wsb, st)
        us.ffn_bwd(p(self.X8), p(self.W1_8), p(self.W2_8), p(self.Z), p(self.H), p(self.G8), p(self.dZ16), p(self.dZ8), p(self.dX),
                   p(self.dW1), p(self.dW2), T, d, f, self.mode, p(self.ws), self.wsb, st)

    def weight_casts(self):
        us, p, st = self.us, self.p, self.torch.cuda.current_stream().cuda_stream
        us.cast_fp8_batch([p(self.W1), p(self.W2)], [p(self.W1_8), p(self.W2_8)], [self.W1.numel(), self.W2.numel()], [us.E4M3, us.E4M3], st)

    def all_casts(self):
        us, p, st = self.us, self.p, self.torch.cuda.current_stream().cuda_stream
        us.cast_fp8_batch([p(self.X), p(self.W1), p(self.W2), p(self.G)], [p(self.X8), p(self.W1_8), p(self.W2_8), p(self.G8)],
                          [self.X.numel(), self.W1.numel(), self.W2.numel(), self.G.numel()], [us.E4M3, us.E4M3, us.E4M3, us.E5M2], st)

    def step_residual(self, tau=0.5):
        """The same step for the residual layer out = sqrt(1-tau) x + sqrt(tau) FFN(x) (interpolation fused into the
        second projection and into grad_X of the first): a side measurement, not `value`."""
        us, p, st = self.us, self.p, self.torch.cuda.current_stream().cuda_stream
        T, d, f = self.T, self.d, self.f
        if self.fp8:
            us.cast_fp8_batch([p(self.X), p(self.W1), p(self.W2), p(self.G)], [p(self.X8), p(self.W1_8), p(self.W2_8), p(self.G8)],
                              [self.X.numel(), self.W1.numel(), self.W2.numel(), self.G.numel()],
                              [us.E4M3, us.E4M3, us.E4M3, us.E5M2], st)
            X, W1, W2, G = self.X8, self.W1_8, self.W2_8, self.G8
        else:
            X, W1, W2, G = self.X, self.W1, self.W2, self.G
        us.ffn_res_fwd(p(self.X), p(X), p(W1), p(W2), p(self.Z), p(self.H), p(self.Y), T, d, f, tau, self.mode, p(self.ws), self.wsb, st)
        us.ffn_res_bwd(p(X), p(W1), p(W2), p(self.Z), p(self.H), p(self.G), p(G), p(self.dZ16), p(self.dZ8), p(self.dX), p(self.dW1),
                       p(self.dW2), T, d, f, tau, self.mode, p(self.ws), self.wsb, st)


    def step_bias(self):
        """The same step for the FFN with bias rows, W2 gelu(W1 x + b1) + b2: biases fused into the two forward epilogues,
        their gradients as column sums of G and of the FP16 dZ (taken inside the epilogue that produces dZ; the FP8 step
        still stores only its E5M2 copy): a side measurement."""
        us, p, st, torch = self.us, self.p, self.torch.cuda.current_stream().cuda_stream, self.torch
        T, d, f = self.T, self.d, self.f
        if not hasattr(self, "b1"):
            self.b1, self.b2 = torch.zeros(f, dtype=torch.float16, device="cuda:0"), torch.zeros(d, dtype=torch.float16, device="cuda:0")
            self.db1, self.db2 = torch.empty_like(self.b1), torch.empty_like(self.b2)
        if self.fp8:
            us.cast_fp8_batch([p(self.X), p(self.W1), p(self.W2), p(self.G)], [p(self.X8), p(self.W1_8), p(self.W2_8), p(self.G8)],
                              [self.X.numel(), self.W1.numel(), self.W2.numel(), self.G.numel()],
                              [us.E4M3, us.E4M3, us.E4M3, us.E5M2], st)
            X, W1, W2, G = self.X8, self.W1_8, self.W2_8, self.G8
        else:
            X, W1, W2, G = self.X, self.W1, self.W2, self.G
        us.ffn_bias_fwd(p(X), p(W1), p(self.b1), p(W2), p(self.b2), p(self.Z), p(self.H), p(self.Y), T, d, f, self.mode, p(self.ws),
                        self.wsb, st)
        us.ffn_bias_bwd(p(X), p(W1), p(W2), p(self.Z), p(self.H), p(G), p(self.G), p(self.dZ16), p(self.dZ8), p(self.dX), p(self.dW1),
                        p(self.dW2), p(self.db1), p(self.db2), T, d, f, self.mode, p(self.ws), self.wsb, st)


class ClockSampler:
    """Samples the GPU's shader clock (the line marked '*' of the driver's pp_dpm_sclk file) from a host thread while a
    measurement runs.  mean() is None when the file cannot be read."""

    def __init__(self, period_s=0.001):
        import glob
        import threading
        self.paths = sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk"))
        self.period, self.samples, self._stop = period_s, [], threading.Event()
        self._thread = threading.Thread(target=self._run, daemon=True)

    def _read(self):
        for path in self.paths:
            try:
                for line in open(path):
                    if "*" in line:
                        return float(line.split(":")[1].lower().split("mhz")[0])
            except (OSError, ValueError, IndexError):
                pass
        return None

    def _run(self):
        while not self._stop.is_set():
            v = self._read()
            if v is not None:
                self.samples.append(v)
            time.sleep(self.period)

    def __enter__(self):
        if self.paths:
            self._thread.start()
        return self

    def __exit__(self, *exc):
        self._stop.set()
        if self.paths:
            self._thread.join()

    def mean(self):
        return sum(self.samples) / len(self.samples) if self.samples else None


def measure_clock(torch, fn, seconds=0.3):
    """Mean shader clock (MHz) while `fn` runs back to back for `seconds` (the timed loop itself can be a few
    milliseconds long, too short for a host-side sampler)."""
    with ClockSampler() as cs:
        t0 = time.perf_counter()
        while time.perf_counter() - t0 < seconds:
            for _ in range(20):
                fn()
            torch.cuda.synchronize()
    return cs.mean(), len(cs.samples)


def ramp_up(torch, fn, seconds=0.15):
    """Untimed: keeps the GPU busy with the step until its clocks have settled.  The first ~30 ms of work
    after an idle period run about 7 % slower than the steady state (measured), which a warm-up of a
    few 0.3 ms steps does not cover."""
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        for _ in range(20):
            fn()
        torch.cuda.synchronize()


def time_steps(torch, fn, steps, warmup):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def time_graph(torch, fn, steps, warmup):
    """Captures one step in a HIP graph (after eager warm-up) and times `steps` replays."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for _ in range(3):
            fn()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        fn()
    for _ in range(warmup):
        graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        graph.replay()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def time_calls(torch, calls, steps):
    """Average duration of each launch of the step, from HIP events on the launch stream.  One call is bracketed
    at a time (the whole step still runs in order, so caches are in the state of a real step): an event pair
    around every launch would put a small bubble between all of them."""
    steps = min(steps, 200)
    res = []
    for i, (name, kind, flop, nbytes, _) in enumerate(calls):
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        torch.cuda.synchronize()
        for s in range(steps):
            for k, c in enumerate(calls):
                if k == i:
                    ev[s][0].record()
                c[4]()
                if k == i:
                    ev[s][1].record()
        torch.cuda.synchronize()
        ms = sum(e0.elapsed_time(e1) for e0, e1 in ev) / steps
        res.append(dict(name=name, kind=kind, ms=ms, flop=flop, bytes=nbytes))
    return res



def pytorch_reference(torch, T, d, f, steps=100, warmup=20):
    """The same FP8 unit-scaled FFN forward + backward written with PyTorch's own ops on the same GPU (FP8 matmuls through
    torch._scaled_mm, i.e. the vendor's GEMM library, casts / GELU / GELU' as eager elementwise kernels, the layout copies
    that interface needs): what a framework-level implementation of the method costs here.  Context, not the target.
    Returns None when this PyTorch build cannot run it."""
    try:
        dev = "cuda:0"
        E4, E5 = torch.float8_e4m3fn, torch.float8_e5m2
        X, W1, W2, G = (torch.randn(s, dtype=torch.float16, device=dev) for s in ((T, d), (d, f), (f, d), (T, d)))
        sc = lambda v: torch.tensor(float(v), device=dev)
        a1, a2, bx2, bx1, bw, one = sc(d ** -0.5), sc(f ** -0.5), sc(d ** -0.5), sc(f ** -0.5), sc(T ** -0.5), sc(1.0)
        ag, bg = 1.7009261846542358, 1.481114387512207

        def mm(a, b_nk, s):       # a [M,K] row-major; b_nk [N,K] row-major, so that b_nk.t() is the column-major [K,N] the call wants
            return torch._scaled_mm(a, b_nk.t(), scale_a=s, scale_b=one, out_dtype=torch.float16)

        def step():
            X8, W1_8, W2_8, G8 = X.to(E4), W1.to(E4), W2.to(E4), G.to(E5)
            Z = mm(X8, W1_8.t().contiguous(), a1)
            H8 = (torch.nn.functional.gelu(Z) * ag).to(E4)
            Y = mm(H8, W2_8.t().contiguous(), a2)
            dH = mm(G8, W2_8, bx2)
            dZ8 = (torch.ops.aten.gelu_backward(dH, Z) * bg).to(E5)
            dW2 = mm(H8.t().contiguous(), G8.t().contiguous(), bw)
            dX = mm(dZ8, W1_8, bx1)
            dW1 = mm(X8.t().contiguous(), dZ8.t().contiguous(), bw)
            return Y, dX, dW1, dW2

        ms_step = time_steps(torch, step, steps, warmup)
        # the six matmuls alone, operands prepared beforehand (a floor for anything built on that library)
        X8, W1_8, W2_8, G8 = X.to(E4), W1.to(E4), W2.to(E4), G.to(E5)
        H8, dZ8 = torch.randn((T, f), device=dev).to(E4), torch.randn((T, f), device=dev).to(E5)
        W1t, W2t, H8t, G8t, X8t, dZ8t = (t.t().contiguous() for t in (W1_8, W2_8, H8, G8, X8, dZ8))

        def gemms():
            mm(X8, W1t, a1); mm(H8, W2t, a2); mm(G8, W2_8, bx2); mm(H8t, G8t, bw); mm(dZ8, W1_8, bx1); mm(X8t, dZ8t, bw)

        ms_gemms = time_steps(torch, gemms, steps, warmup)
        flop = 12.0 * T * d * f
        return {"what": "FP8 unit-scaled FFN fwd+bwd with PyTorch ops on this GPU (torch._scaled_mm + eager elementwise kernels and "
                        "layout copies); six_matmuls_only: the vendor library's six FP8 matmuls with operands prepared beforehand",
                "ms_per_step": ms_step, "TFLOPs": flop / (ms_step * 1e-3) * 1e-12,
                "six_matmuls_only_ms": ms_gemms, "six_matmuls_only_TFLOPs": flop / (ms_gemms * 1e-3) * 1e-12}
    except Exception as e:          # an op or type this build lacks: the comparison is simply left out
        return {"unavailable": repr(e)[:200]}

def range_stress(torch, us, steps=30):
    """Config "FP8 range-stress GEMM sweep": square M = N = K in {2048, 4096, 8192}; X and W are N(0,1) in FP32 with one entry
    in 1000 replaced by +-1000; each run is a scaled cast of both operands to E4M3 (s = 1) followed by the matmul with
    alpha = K^-1/2.  Timed with the operands resident in HBM; the matmul alone and the cast + matmul run."""
    dev, st = "cuda:0", torch.cuda.current_stream().cuda_stream
    out = {}
    for N in (2048, 4096, 8192):
        g = torch.Generator(device=dev)
        g.manual_seed(20230314 + N)
        ops = []
        for _ in range(2):
            a = torch.randn((N, N), generator=g, device=dev, dtype=torch.float32)
            hit = torch.rand((N, N), generator=g, device=dev) < 1e-3
            sign = torch.where(torch.rand((N, N), generator=g, device=dev) < 0.5, -1000.0, 1000.0)
            ops.append(torch.where(hit, sign, a))
        X8, W8 = (torch.empty((N, N), dtype=torch.uint8, device=dev) for _ in range(2))
        Y = torch.empty((N, N), dtype=torch.float16, device=dev)
        stats = torch.zeros(4, dtype=torch.int64, device=dev)

        def casts():
            us.cast_fp8(ops[0].data_ptr(), us.F32, X8.data_ptr(), us.E4M3, N * N, 1.0, stats.data_ptr(), st)
            us.cast_fp8(ops[1].data_ptr(), us.F32, W8.data_ptr(), us.E4M3, N * N, 1.0, stats.data_ptr(), st)

        def gemm():
            us.linear_fwd(X8.data_ptr(), W8.data_ptr(), Y.data_ptr(), N, N, N, us.E4M3, us.E4M3, us.F16, 0.0, us.EPI_NONE, 0.0, None, None, None, 0, st)

        def both():
            casts()
            gemm()
        casts()
        ramp_up(torch, gemm, 0.05)
        ms_g = time_steps(torch, gemm, steps, 5)
        ms_b = time_steps(torch, both, steps, 5)
        ms_c = time_steps(torch, casts, steps, 5)
        flop = 2.0 * N ** 3
        out[str(N)] = {"matmul_ms": ms_g, "matmul_TFLOPs": flop / (ms_g * 1e-3) * 1e-12, "frac_of_mfma_peak": flop / (ms_g * 1e-3) * 1e-12 / PEAK_TFLOPS["fp8"],
                       "cast_plus_matmul_ms": ms_b, "cast_plus_matmul_TFLOPs": flop / (ms_b * 1e-3) * 1e-12,
                       "casts_GBps": 2 * 5.0 * N * N / (ms_c * 1e-3) * 1e-9, "kernel": us.last_launch()}
        del ops, X8, W8, Y
    out["what"] = "scaled cast FP32 -> E4M3 (5 B / element, with counters) of both operands, then Y = K^-1/2 X W; N(0,1) with 0.1 % +-1000 outliers"
    return out


def cpu_baseline(ffn, sample_tokens):
    """The oracle, as it stands, on the first `sample_tokens` tokens of the same tensors (all of d and f)."""
    import numpy as np
    import oracle
    n = sample_tokens
    X = ffn.X[:n].cpu().numpy()
    G = ffn.G[:n].cpu().numpy()
    W1, W2 = ffn.W1.cpu().numpy(), ffn.W2.cpu().numpy()
    t0 = time.perf_counter()
    fw = oracle.ffn_fwd(X, W1, W2, ffn.fp8)
    oracle.ffn_bwd(X, W1, W2, G, fw, ffn.fp8)
    dt = time.perf_counter() - t0
    flop = 12.0 * n * ffn.d * ffn.f
    return dict(value=flop / dt * 1e-12, unit="TFLOP/s", cores=oracle.cpu_threads(), kind="oracle", seconds=dt,
                sample=f"first {n} of {ffn.T} tokens, full d_model and d_ff, every stage ({'casts, ' if ffn.fp8 else ''}6 matmuls, GELU fwd/bwd)")


def cpu_range_stress(N=2048):
    """The oracle on one run of the range-stress sweep: both scaled casts (FP32 -> E4M3 with counters) and the product."""
    import numpy as np
    import oracle
    import synth
    seed = synth.C4_SEED + N
    ops = [synth.place_outliers(synth.normal(seed, t, (N, N), 1.0, np.float32), 1.0, synth.outlier_positions(seed, t, N * N))
           for t in (synth.T_X, synth.T_W1)]
    t0 = time.perf_counter()
    codes = [oracle.cast_fp8(a, oracle.E4M3, 1.0)[0] for a in ops]
    oracle.linear_fwd(codes[0], codes[1], float(N) ** -0.5, oracle.E4M3, oracle.E4M3)
    dt = time.perf_counter() - t0
    return dict(value=2.0 * N ** 3 / dt * 1e-12, unit="TFLOP/s", cores=oracle.cpu_threads(), kind="oracle", seconds=dt,
                sample=f"range stress, M = N = K = {N}, sigma = 1, s = 1: two casts with counters and the matmul")


def measured_traffic(workload):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary (None if absent)."""
    path = os.path.join(ROOT, "profiles", f"ffn_bwd_layer2_{workload.lower()}_hbm_traffic.md")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="C3", choices=sorted(WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--graph", action="store_true", help="time HIP-graph replays of the captured step instead of eager launches")
    ap.add_argument("--no-secondary", action="store_true", help="skip the FP16 BERT-base side measurement")
    ap.add_argument("--cpu-sample-tokens", type=int, default=0, help="tokens the oracle is timed on (0: all of the workload's, capped at 8192)")
    ap.add_argument("--vendor-reference", action="store_true",
                    help="also time the same FFN written with PyTorch ops / the vendor's FP8 GEMM (context; off by default)")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run one plain 256 MiB FP16 copy kernel (y = x + 0): the known-size reference for scaling "
                         "the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (the path would shard over tokens with one all-reduce of the weight "
              "gradients; that is not built); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2303_11257_amd as us
    import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    us.lib()   # fails loudly if the HIP library is not built
    torch.cuda.set_device(0)

    if args.pmc_calibration:
        x = torch.ones(128 << 20, dtype=torch.float16, device="cuda:0")     # 256 MiB read + 256 MiB written
        y = torch.empty_like(x)
        torch.add(x, 0, out=y)
        torch.cuda.synchronize()
        del x, y

    w = WORKLOADS[args.workload]
    ffn = Ffn(torch, us, synth, w["T"], w["d"], w["f"], w["fp8"], synth.BASE_SEED + 2)
    ramp_up(torch, ffn.step)
    ms_eager = time_steps(torch, ffn.step, args.steps, args.warmup)
    # eager launches already run back to back (the host stays ahead); a HIP-graph replay of the same
    # step is available for comparison and measures the same within noise
    ms_step = time_graph(torch, ffn.step, args.steps, args.warmup) if args.graph else ms_eager
    tflops = ffn.flop / (ms_step * 1e-3) * 1e-12
    dt_key = "fp8" if w["fp8"] else "f16"

    clock_mhz, clock_samples = measure_clock(torch, ffn.step)
    per_call = time_calls(torch, ffn.calls(), args.steps)
    gemms = [c for c in per_call if c["kind"] == "gemm"]
    casts = [c for c in per_call if c["kind"] == "cast"]
    dom = max(gemms, key=lambda c: c["ms"])
    gemm_ms = sum(c["ms"] for c in gemms)
    roof = dict(bound="mfma", kernel=dom["name"], achieved=dom["flop"] / (dom["ms"] * 1e-3) * 1e-12,
                peak=PEAK_TFLOPS[dt_key], unit="TFLOP/s", traffic=measured_traffic(args.workload))
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["ms"] = dom["ms"]
    if clock_mhz:
        # the published peak is at the nominal 2400 MHz; under MFMA load the chip runs below it (power)
        roof["shader_clock_mhz"] = clock_mhz
        roof["peak_at_measured_clock"] = roof["peak"] * clock_mhz / 2400.0
        roof["frac_at_measured_clock"] = roof["achieved"] / roof["peak_at_measured_clock"]
    roof["all_gemms_achieved"] = sum(c["flop"] for c in gemms) / (gemm_ms * 1e-3) * 1e-12
    out = {
        "metric": "unit-scaled FFN fwd+bwd TFLOP/s",
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "fp8" if w["fp8"] else "f16", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {w['desc']}", "tokens": w["T"], "d_model": w["d"], "d_ff": w["f"],
                   "step": "one batched cast of X,W1,W2,G + Linear+GELU + Linear + 4 backward matmuls (GELU' fused; stored: Z16, H8, Y16, dZ8, dX16, dW16)" if w["fp8"]
                           else "Linear+GELU + Linear + 4 backward matmuls (GELU' fused)"},
        "frac_of_mfma_peak": tflops / PEAK_TFLOPS[dt_key],
        "shader_clock": {"mhz_during_the_step_loop": clock_mhz, "samples": clock_samples, "nominal_mhz": 2400.0,
                         "frac_of_mfma_peak_at_measured_clock": (tflops / (PEAK_TFLOPS[dt_key] * clock_mhz / 2400.0)) if clock_mhz else None,
                         "how": "pp_dpm_sclk sampled every ms from a host thread while the step runs back to back for 0.3 s"},
        "launch": "hip-graph replay of the captured step" if args.graph else "eager",
        "roofline": roof,
        "calls_ms": {c["name"]: round(c["ms"], 5) for c in per_call},
        "calls_tflops": {c["name"]: round(c["flop"] / (c["ms"] * 1e-3) * 1e-12, 1) for c in gemms},
    }
    if casts:
        # kernel rate: the batched cast launched back to back (launch gaps hidden by the queue), which is what rocprofv3
        # reports as the kernel's duration; the in-step figure brackets ONE launch with events inside the running step
        # and so includes the gap to the neighbouring launches
        cb, cm = sum(c["bytes"] for c in casts), sum(c["ms"] for c in casts)
        ms_k = time_steps(torch, ffn.all_casts, max(args.steps, 50), 10)
        out["cast"] = {"GBps": cb / (ms_k * 1e-3) * 1e-9, "frac_of_hbm_peak": cb / (ms_k * 1e-3) * 1e-9 / PEAK_HBM_GBS,
                       "ms_back_to_back": ms_k, "bytes_per_elem": 3, "bytes_per_launch": cb,
                       "in_step_event_bracket": {"ms": cm, "GBps": cb / (cm * 1e-3) * 1e-9,
                                                 "what": "events around the one cast launch inside the step: includes the launch gap"}}
        ms_act = time_steps(torch, ffn.step_act_casts_only, args.steps, args.warmup)
        ms_wc = time_steps(torch, ffn.weight_casts, max(args.steps, 50), 10)
        out["step_with_activation_and_gradient_casts_only"] = {
            "what": "the step with the E4M3 weights reused (gradient accumulation: the weights change once per many micro-batches); "
                    "the weight casts are their own figure",
            "ms_per_step": ms_act, "TFLOPs": ffn.flop / (ms_act * 1e-3) * 1e-12,
            "frac_of_mfma_peak": ffn.flop / (ms_act * 1e-3) * 1e-12 / PEAK_TFLOPS[dt_key],
            "weight_casts_ms": ms_wc, "weight_casts_GBps": 3.0 * (ffn.W1.numel() + ffn.W2.numel()) / (ms_wc * 1e-3) * 1e-9}
        out["gemm_kernels_only"] = {"ms": gemm_ms, "TFLOPs": roof["all_gemms_achieved"], "frac_of_mfma_peak": roof["all_gemms_achieved"] / PEAK_TFLOPS[dt_key],
                                    "what": "sum of the four matmul launches' event-bracketed durations inside the step"}
    if not args.no_secondary:
        ms_res = time_steps(torch, ffn.step_residual, args.steps, args.warmup)
        out["residual_layer"] = {"what": "same workload with the fixed(tau=0.5) residual interpolation fused into the step "
                                         "(forward output and grad_X read one more FP16 [tokens, d_model] tensor each)",
                                 "ms_per_step": ms_res, "TFLOPs": ffn.flop / (ms_res * 1e-3) * 1e-12}
        ms_b = time_steps(torch, ffn.step_bias, args.steps, args.warmup)
        out["ffn_with_biases"] = {"what": "same workload with bias rows b1, b2 (added in the forward epilogues) and their gradients "
                                          "(column sums of G, and of the FP16 dZ inside the GELU' epilogue)",
                                  "ms_per_step": ms_b, "TFLOPs": ffn.flop / (ms_b * 1e-3) * 1e-12}
    if not args.no_secondary:
        # stand-alone elementwise kernels (HBM bound): 256 Mi FP16 elements (512 MB per tensor: twice the 256 MB last-level
        # cache, so the rates are HBM's), algorithmic bytes 4 B (forward) / 6 B (backward) / 6 B (add)
        n = 256 << 20
        za, zb, zo = (torch.randn(n, dtype=torch.float16, device="cuda:0") for _ in range(3))
        st = torch.cuda.current_stream().cuda_stream
        ew = {}
        for name, kind in (("gelu", us.ACT_GELU), ("relu", us.ACT_RELU), ("tanh", us.ACT_TANH), ("sigmoid", us.ACT_SIGMOID)):
            ms = time_steps(torch, lambda: us.act_fwd(za.data_ptr(), zo.data_ptr(), n, us.F16, kind, 0.0, 0.0, st), 20, 3)
            ew[name + "_fwd_GBps"] = round(4.0 * n / (ms * 1e-3) * 1e-9, 1)
            ms = time_steps(torch, lambda: us.act_bwd(za.data_ptr(), zb.data_ptr(), zo.data_ptr(), n, us.F16, kind, 0.0, 0.0, st), 20, 3)
            ew[name + "_bwd_GBps"] = round(6.0 * n / (ms * 1e-3) * 1e-9, 1)
        ms = time_steps(torch, lambda: us.weighted_add(za.data_ptr(), zb.data_ptr(), zo.data_ptr(), n, us.F16, 0.8, 0.6, st), 20, 3)
        ew["weighted_add_GBps"] = round(6.0 * n / (ms * 1e-3) * 1e-9, 1)
        # scaled layer norm on [262144, 1024] FP16 (the BERT-large hidden size): 4 B / element forward, 6 B backward
        lb, ln = n // 1024, 1024
        lw, lc, ldw, ldc = (torch.ones(ln, dtype=torch.float16, device="cuda:0") for _ in range(4))
        lwsb = us.layer_norm_workspace_bytes(lb, ln)
        lws = torch.empty(lwsb, dtype=torch.uint8, device="cuda:0")
        ms = time_steps(torch, lambda: us.layer_norm_fwd(za.data_ptr(), lw.data_ptr(), lc.data_ptr(), zo.data_ptr(), lb, ln, 1e-5, st), 20, 3)
        ew["layer_norm_fwd_GBps"] = round(4.0 * n / (ms * 1e-3) * 1e-9, 1)
        ms = time_steps(torch, lambda: us.layer_norm_bwd(za.data_ptr(), lw.data_ptr(), zb.data_ptr(), zo.data_ptr(), ldw.data_ptr(),
                                                         ldc.data_ptr(), lb, ln, 1e-5, 0.0, lws.data_ptr(), lwsb, st), 20, 3)
        ew["layer_norm_bwd_GBps"] = round(6.0 * n / (ms * 1e-3) * 1e-9, 1)
        bwsb = us.bias_grad_workspace_bytes(lb, ln)
        bws = torch.empty(bwsb, dtype=torch.uint8, device="cuda:0")
        ms = time_steps(torch, lambda: us.bias_grad(za.data_ptr(), us.F16, ldc.data_ptr(), lb, ln, 0.0, bws.data_ptr(), bwsb, st), 20, 3)
        ew["bias_grad_GBps"] = round(2.0 * n / (ms * 1e-3) * 1e-9, 1)
        # scaled softmax on [524288, 512] (attention rows): 4 B / element forward, 6 B backward; cross-entropy on
        # [8192, 30528] (a BERT vocabulary, padded to a multiple of 8): loss and gradient, 4 B / element
        sb, ss = n // 512, 512
        ms = time_steps(torch, lambda: us.softmax_fwd(za.data_ptr(), zo.data_ptr(), sb, ss, 0.0, 0.0, st), 20, 3)
        ew["softmax_fwd_GBps"] = round(4.0 * n / (ms * 1e-3) * 1e-9, 1)
        ms = time_steps(torch, lambda: us.softmax_bwd(za.data_ptr(), zb.data_ptr(), zo.data_ptr(), sb, ss, 0.0, 0.0, st), 20, 3)
        ew["softmax_bwd_GBps"] = round(6.0 * n / (ms * 1e-3) * 1e-9, 1)
        xr, xs = 8192, 30528                      # the tokens of the C3 batch against a BERT vocabulary
        xa = torch.randn((xr, xs), dtype=torch.float16, device="cuda:0")
        xo = torch.empty_like(xa)
        xt = torch.randint(0, xs, (xr,), dtype=torch.int32, device="cuda:0")
        xl = torch.empty(xr, dtype=torch.float32, device="cuda:0")
        ms = time_steps(torch, lambda: us.softmax_xent(xa.data_ptr(), xt.data_ptr(), xl.data_ptr(), xo.data_ptr(), xr, xs, 0.0, 0.0, st), 20, 3)
        del xa, xo
        ew["softmax_xent_GBps"] = round(4.0 * xr * xs / (ms * 1e-3) * 1e-9, 1)
        ms = time_steps(torch, lambda: us.sum_fwd(za.data_ptr(), zo.data_ptr(), sb, ss, 0.0, st), 20, 3)
        ew["sum_fwd_GBps"] = round(2.0 * n / (ms * 1e-3) * 1e-9, 1)
        # diagnostics: read-only, 2 B / element
        hist = torch.zeros(us.HIST_BINS, dtype=torch.int64, device="cuda:0")
        sums = torch.zeros(2, dtype=torch.float64, device="cuda:0")
        ms = time_steps(torch, lambda: us.exponent_histogram(za.data_ptr(), us.F16, n, hist.data_ptr(), st), 20, 3)
        ew["exponent_histogram_GBps"] = round(2.0 * n / (ms * 1e-3) * 1e-9, 1)
        ms = time_steps(torch, lambda: us.cast_snr(za.data_ptr(), us.F16, n, us.E4M3, 1.0, sums.data_ptr(), st), 20, 3)
        ew["cast_snr_GBps"] = round(2.0 * n / (ms * 1e-3) * 1e-9, 1)
        ew["snr_e4m3_unit_normal"] = round(float(sums[0] / sums[1]), 1)
        # the same two on a tensor that fits the last-level cache (32 Mi elements): fixed costs show
        ns = 32 << 20
        ms = time_steps(torch, lambda: us.exponent_histogram(za.data_ptr(), us.F16, ns, hist.data_ptr(), st), 20, 3)
        ew["exponent_histogram_64MB_GBps"] = round(2.0 * ns / (ms * 1e-3) * 1e-9, 1)
        ew["peak_GBps"] = PEAK_HBM_GBS
        out["elementwise"] = ew
        del za, zb, zo
    if not args.no_secondary:
        # unit-scaled attention (unfused: batched matmuls + scaled softmax), 16 sequences x 16 heads, 512 tokens, head size 64
        ah, as_, ad = 256, 512, 64
        e16 = lambda *shape: torch.randn(shape, dtype=torch.float16, device="cuda:0")
        aq, ak, av, ado = (e16(ah, as_, ad) for _ in range(4))
        aA, aP, adP, adA = (torch.empty((ah, as_, as_), dtype=torch.float16, device="cuda:0") for _ in range(4))
        aO, adQ, adK, adV = (torch.empty((ah, as_, ad), dtype=torch.float16, device="cuda:0") for _ in range(4))
        st = torch.cuda.current_stream().cuda_stream
        dp = lambda t: t.data_ptr()

        def attn_step():
            us.attention_fwd(dp(aq), dp(ak), dp(av), dp(aA), dp(aP), dp(aO), ah, as_, ad, st)
            us.attention_bwd(dp(aq), dp(ak), dp(av), dp(aA), dp(aP), dp(ado), dp(adP), dp(adA), dp(adQ), dp(adK), dp(adV), ah, as_, ad, st)
        ms_a = time_steps(torch, attn_step, 20, 3)
        a_flop = 12.0 * as_ * as_ * ad * ah
        # [heads, s, s] tensors: A written + read twice, P written + read twice, dP written + read, dA written + read twice
        a_bytes = 11.0 * ah * as_ * as_ * 2
        out["attention"] = {"what": "unit-scaled attention fwd+bwd, FP16, 256 heads x 512 tokens x 64, unfused (6 batched matmuls, "
                                    "scaled softmax fwd and bwd; scores and probabilities stored)",
                            "ms_per_step": ms_a, "TFLOPs": a_flop / (ms_a * 1e-3) * 1e-12,
                            "score_tensor_GBps": a_bytes / (ms_a * 1e-3) * 1e-9}
        del aq, ak, av, ado, aA, aP, adP, adA, aO, adQ, adK, adV
    if args.vendor_reference and w["fp8"]:
        out["pytorch_reference"] = pytorch_reference(torch, w["T"], w["d"], w["f"])
    if not args.no_secondary:
        out["range_stress"] = range_stress(torch, us)
    if not args.no_secondary and args.workload != "C2":
        w2 = WORKLOADS["C2"]
        f2 = Ffn(torch, us, synth, w2["T"], w2["d"], w2["f"], False, synth.BASE_SEED + 1)
        ramp_up(torch, f2.step)
        ms2 = time_graph(torch, f2.step, args.steps, args.warmup) if args.graph else time_steps(torch, f2.step, args.steps, args.warmup)
        t2 = f2.flop / (ms2 * 1e-3) * 1e-12
        out["fp16_bert_base"] = {"workload": "C2: " + w2["desc"], "ms_per_step": ms2, "TFLOPs": t2,
                                 "frac_of_mfma_peak": t2 / PEAK_TFLOPS["f16"]}
        if not args.no_cpu_baseline:
            out["fp16_bert_base"]["cpu_baseline"] = cpu_baseline(f2, w2["T"])
        del f2
    if not args.no_secondary and args.workload == "C3":
        # the same step at a size where the main loops dominate (reduction lengths 4096 / 16384 / 32768)
        w5 = WORKLOADS["C5"]
        f5 = Ffn(torch, us, synth, w5["T"], w5["d"], w5["f"], True, synth.BASE_SEED + 4)
        ramp_up(torch, f5.step)
        ms5 = time_steps(torch, f5.step, 10, 2)
        t5 = f5.flop / (ms5 * 1e-3) * 1e-12
        out["fp8_large"] = {"workload": "C5: " + w5["desc"], "ms_per_step": ms5, "TFLOPs": t5, "frac_of_mfma_peak": t5 / PEAK_TFLOPS["fp8"]}
        if not args.no_cpu_baseline:
            out["fp8_large"]["cpu_baseline"] = cpu_baseline(f5, 256)
        del f5
    if not args.no_cpu_baseline and not args.no_secondary:
        out["range_stress"]["cpu_baseline"] = cpu_range_stress(2048)
    if not args.no_cpu_baseline:
        n_cpu = args.cpu_sample_tokens if args.cpu_sample_tokens > 0 else min(w["T"], 8192)
        out["cpu_baseline"] = cpu_baseline(ffn, min(n_cpu, w["T"]))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
