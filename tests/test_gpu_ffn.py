"""GPU parity for the whole FFN path (cast -> Linear+GELU -> Linear, and its backward) through
us_ffn_fwd / us_ffn_bwd: full comparison on a small ragged shape, sampled rows / columns at the
benchmark shapes.  Every stage is compared with the oracle applied to the GPU's own stored inputs of
that stage."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2303_11257_amd as us
import synth
from gpu_util import DEV, assert_close, ptr, stream, to_dev, to_np

pytestmark = pytest.mark.gpu


class FfnRun:
    """Device buffers of one FFN forward + backward; `dev` tensors stay on the GPU."""

    def __init__(self, X, W1, W2, G, fp8, store_dz16=True, prebuilt_tables=False):
        self.fp8 = fp8
        T, d = X.shape
        f = W1.shape[1]
        self.T, self.d, self.f = T, d, f
        dev = {k: (v if isinstance(v, torch.Tensor) else to_dev(v)) for k, v in dict(X=X, W1=W1, W2=W2, G=G).items()}
        st = stream()
        if fp8:
            for k, fmt in (("X", us.E4M3), ("W1", us.E4M3), ("W2", us.E4M3), ("G", us.E5M2)):
                dst = torch.empty(dev[k].shape, dtype=torch.uint8, device=DEV)
                us.cast_fp8(ptr(dev[k]), us.F16, ptr(dst), fmt, dev[k].numel(), 1.0, None, st)
                dev[k + "op"] = dst
        else:
            for k in ("X", "W1", "W2", "G"):
                dev[k + "op"] = dev[k]
        e = lambda shape, dt=torch.float16: torch.empty(shape, dtype=dt, device=DEV)
        dev["Z"], dev["Y"] = e((T, f)), e((T, d))
        dev["H"] = e((T, f), torch.uint8 if fp8 else torch.float16)
        dev["dZ16"], dev["dX"], dev["dW1"], dev["dW2"] = e((T, f)), e((T, d)), e((d, f)), e((f, d))
        dev["dZ8"] = e((T, f), torch.uint8) if fp8 else None
        if not store_dz16:
            dev["dZ16"] = None                     # FP8 only: the layer-1 matmuls read the E5M2 codes
        wsb = us.ffn_workspace_bytes(T, d, f)
        ws = torch.full((max(wsb, 16),), 0xA5, dtype=torch.uint8, device=DEV)
        mode = us.FFN_FP8 if fp8 else 0
        if prebuilt_tables:                       # tables once, then calls that must leave them alone
            us.gelu_tables(ptr(ws), wsb, 0.0, 0.0, st)
            mode |= us.FFN_TABLES_READY
            tables = ws[:us.TABLE_AREA_BYTES].clone()
        us.ffn_fwd(ptr(dev["Xop"]), ptr(dev["W1op"]), ptr(dev["W2op"]), ptr(dev["Z"]), ptr(dev["H"]), ptr(dev["Y"]),
                   T, d, f, mode, ptr(ws), wsb, st)
        us.ffn_bwd(ptr(dev["Xop"]), ptr(dev["W1op"]), ptr(dev["W2op"]), ptr(dev["Z"]), ptr(dev["H"]), ptr(dev["Gop"]),
                   ptr(dev["dZ16"]), ptr(dev["dZ8"]), ptr(dev["dX"]), ptr(dev["dW1"]), ptr(dev["dW2"]), T, d, f, mode,
                   ptr(ws), wsb, st)
        torch.cuda.synchronize()
        if prebuilt_tables:
            assert torch.equal(ws[:us.TABLE_AREA_BYTES], tables), "the calls wrote into the table area"
        self.dev = dev

    def rows(self, name, idx):
        return self.dev[name][torch.as_tensor(idx, device=DEV)].cpu().numpy()

    def cols(self, name, idx):
        return self.dev[name][:, torch.as_tensor(idx, device=DEV)].contiguous().cpu().numpy()

    def full(self, name):
        return self.dev[name].cpu().numpy()


def check_ffn(run: FfnRun, rows, cols_f, cols_d, dw1_cols=None):
    """rows: token rows (sampled, or a slab); cols_f / cols_d: indices in the f and d dimensions whose rows of dW2 / dW1
    are compared over all tokens; dw1_cols: columns of dW1 (indices in f) compared over all of d and all tokens."""
    fp8, T, d, f = run.fp8, run.T, run.d, run.f
    act, grad = (O.E4M3, O.E5M2) if fp8 else (O.F16, O.F16)
    ag, bg = O.gelu_scales()
    a1, bx1, bw1 = O.linear_scales(T, d, f)
    a2, bx2, bw2 = O.linear_scales(T, f, d)
    W1, W2 = run.full("W1op"), run.full("W2op")
    X_r, G_r = run.rows("Xop", rows), run.rows("Gop", rows)
    if fp8:   # operands were produced by the GPU cast: bit exact against the oracle cast of the FP16 tensors
        assert np.array_equal(X_r, O.cast_fp8(run.rows("X", rows), O.E4M3)[0])
        assert np.array_equal(G_r, O.cast_fp8(run.rows("G", rows), O.E5M2)[0])
        assert np.array_equal(W1, O.cast_fp8(run.full("W1"), O.E4M3)[0])
    errs = {}
    # forward, layer 1 + fused GELU
    Z_r = run.rows("Z", rows)
    errs["Z"] = assert_close(Z_r, O.linear_fwd(X_r, W1, a1, act, act), "Z", fp8=fp8)
    H_ref16 = O.gelu_fwd(Z_r, ag)
    H_r = run.rows("H", rows)
    if fp8:
        # only the codes are stored: they may differ from cast(oracle GELU of the stored Z) by one code
        # where the FP32 GELU moved the FP16 value across an FP8 rounding boundary
        ref8 = O.cast_fp8(H_ref16, O.E4M3)[0]
        diff = np.abs(H_r.astype(np.int32) - ref8.astype(np.int32))
        assert diff.max() <= 1 and np.mean(diff != 0) < 1e-3
    else:
        errs["H"] = assert_close(H_r, H_ref16, "H")
    # forward, layer 2 (its operand is the GPU's own stored H)
    errs["Y"] = assert_close(run.rows("Y", rows), O.linear_fwd(H_r, W2, a2, act, act), "Y", fp8=fp8)
    # backward, layer 2: dH (not stored) -> dZ
    dH_ref = O.linear_bwd_dx(G_r, W2, bx2, grad, act)
    dZ_r = run.rows("dZ16", rows)
    errs["dZ"] = assert_close(dZ_r, O.gelu_bwd(Z_r, dH_ref, bg), "dZ", fp8=fp8)
    if fp8:
        dZ8_r = run.rows("dZ8", rows)
        assert np.array_equal(dZ8_r, O.cast_fp8(dZ_r, O.E5M2)[0])         # FP8 copy of the stored FP16 dZ: bit exact
    dZop_r = run.rows("dZ8", rows) if fp8 else dZ_r
    errs["dX"] = assert_close(run.rows("dX", rows), O.linear_bwd_dx(dZop_r, W1, bx1, grad, act), "dX", fp8=fp8)
    # weight gradients: all tokens, sampled output rows (= sampled columns of the left operand)
    H_c = run.cols("H", cols_f)                                            # [T, |cols_f|]
    G_all = run.full("Gop")
    errs["dW2"] = assert_close(run.rows("dW2", cols_f), O.linear_bwd_dw(H_c, G_all, bw2, act, grad), "dW2", fp8=fp8)
    X_c = run.cols("Xop", cols_d)
    dZ_all = run.full("dZ8" if fp8 else "dZ16")
    errs["dW1"] = assert_close(run.rows("dW1", cols_d), O.linear_bwd_dw(X_c, dZ_all, bw1, act, grad), "dW1", fp8=fp8)
    if dw1_cols is not None:
        dZ_c = np.ascontiguousarray(dZ_all[:, dw1_cols])
        errs["dW1 columns"] = assert_close(run.cols("dW1", dw1_cols), O.linear_bwd_dw(run.full("Xop"), dZ_c, bw1, act, grad),
                                           "dW1 columns", fp8=fp8)
    return errs


def check_sampled_elements(run: FfnRun, count, seed):
    """`count` uniformly drawn elements of every stored tensor, each against the oracle's value for that one element (a
    1 x 1 product over the full reduction length on the GPU's own stored operands): reaches tiles that no slab meets."""
    fp8, T, d, f = run.fp8, run.T, run.d, run.f
    act, grad = (O.E4M3, O.E5M2) if fp8 else (O.F16, O.F16)
    ag, bg = O.gelu_scales()
    a1, bx1, bw1 = O.linear_scales(T, d, f)
    a2, bx2, bw2 = O.linear_scales(T, f, d)
    rng = np.random.default_rng(seed)
    dev = run.dev
    dZop = dev["dZ8"] if fp8 else dev["dZ16"]

    def pick(rows_of, cols_of):
        return torch.as_tensor(rng.integers(0, rows_of, count), device=DEV), torch.as_tensor(rng.integers(0, cols_of, count), device=DEV)

    def at(t, i, j):
        return t[i, j].cpu().numpy()

    def each(fn, A, B):          # A[s] and B[s]: the two vectors of element s, as [count, K] arrays
        A, B = A.cpu().numpy(), B.cpu().numpy()
        return np.array([fn(A[s:s + 1], B[s:s + 1]) for s in range(count)])

    # Z[i, j] = a1 X[i, :] . W1[:, j]      (the grad_X form of the oracle takes both vectors as rows)
    i, j = pick(T, f)
    Zs = at(dev["Z"], i, j)
    ref = each(lambda x, w: O.linear_bwd_dx(x, w, a1, act, act)[0, 0], dev["Xop"][i], dev["W1op"][:, j].t().contiguous())
    assert_close(Zs, ref, "Z elements", fp8=fp8)
    # Y[i, j] = a2 H[i, :] . W2[:, j]
    i, j = pick(T, d)
    ref = each(lambda h, w: O.linear_bwd_dx(h, w, a2, act, act)[0, 0], dev["H"][i], dev["W2op"][:, j].t().contiguous())
    assert_close(at(dev["Y"], i, j), ref, "Y elements", fp8=fp8)
    # dZ[i, j] = gelu'(Z[i, j]) * fp16(bx2 G[i, :] . W2[j, :])
    i, j = pick(T, f)
    dH = each(lambda g, w: O.linear_bwd_dx(g, w, bx2, grad, act)[0, 0], dev["Gop"][i], dev["W2op"][j])
    ref = O.gelu_bwd(at(dev["Z"], i, j), dH.astype(np.float16), bg)
    if dev["dZ16"] is not None:
        assert_close(at(dev["dZ16"], i, j), ref, "dZ elements", fp8=fp8)
    # dX[i, k] = bx1 dZ[i, :] . W1[k, :]
    i, k = pick(T, d)
    ref = each(lambda g, w: O.linear_bwd_dx(g, w, bx1, grad, act)[0, 0], dZop[i], dev["W1op"][k])
    assert_close(at(dev["dX"], i, k), ref, "dX elements", fp8=fp8)
    # dW2[k, j] = bw2 H[:, k] . G[:, j];  dW1[k, j] = bw1 X[:, k] . dZ[:, j]      (sums over all tokens)
    k, j = pick(f, d)
    ref = each(lambda h, g: O.linear_bwd_dw(h.T, g.T, bw2, act, grad)[0, 0], dev["H"][:, k].t().contiguous(), dev["Gop"][:, j].t().contiguous())
    assert_close(at(dev["dW2"], k, j), ref, "dW2 elements", fp8=fp8)
    k, j = pick(d, f)
    ref = each(lambda x, g: O.linear_bwd_dw(x.T, g.T, bw1, act, grad)[0, 0], dev["Xop"][:, k].t().contiguous(), dZop[:, j].t().contiguous())
    assert_close(at(dev["dW1"], k, j), ref, "dW1 elements", fp8=fp8)


@pytest.mark.parametrize("fp8", [False, True])
def test_small_ragged_ffn_full_comparison(fp8):
    T, d, f = 272, 144, 400
    X, W1, W2, G = synth.ffn_inputs(T, d, f, seed=127)
    run = FfnRun(X, W1, W2, G, fp8)
    check_ffn(run, np.arange(T), np.arange(f), np.arange(d))


def _same_without_fp16_dz(run, X, W1, W2, G):
    """FP8 step that does not store the FP16 dZ, with the GELU tables built once beforehand instead of
    inside the calls: every other output is bit-identical."""
    lean = FfnRun(X, W1, W2, G, fp8=True, store_dz16=False, prebuilt_tables=True)
    for name in ("Z", "H", "Y", "dZ8", "dX", "dW1", "dW2"):
        assert torch.equal(lean.dev[name], run.dev[name]), name


def test_fp8_ffn_without_fp16_dz_small():
    T, d, f = 272, 144, 400
    X, W1, W2, G = synth.ffn_inputs(T, d, f, seed=127)
    _same_without_fp16_dz(FfnRun(X, W1, W2, G, fp8=True), X, W1, W2, G)



@pytest.mark.parametrize("fp8", [False, True])
def test_end_to_end_drift_against_the_oracle_chain(fp8, record_property):
    """The stage-wise comparisons above feed every oracle stage with the GPU's own stored inputs.  Here the oracle runs
    its whole chain by itself and the final tensors are compared: intermediate rounding flips (FP16 steps, FP8 codes at
    a boundary) now propagate, so this drift is reported (RMS and maximum, relative to the unit scale of the tensors)
    and only loosely gated."""
    T, d, f = 1024, 256, 1040
    X, W1, W2, G = synth.ffn_inputs(T, d, f, seed=131)
    run = FfnRun(X, W1, W2, G, fp8)
    fw = O.ffn_fwd(X, W1, W2, fp8)
    bw = O.ffn_bwd(X, W1, W2, G, fw, fp8)
    ref = dict(Z=fw["Z"], Y=fw["Y"], dZ16=bw["dZ"], dX=bw["dX"], dW1=bw["dW1"], dW2=bw["dW2"])
    for name, r in ref.items():
        g = run.full(name).astype(np.float64)
        e = g - r.astype(np.float64)
        rms, mx = float(np.sqrt(np.mean(e * e))), float(np.abs(e).max())
        record_property(f"drift_{name}_rms", rms)
        record_property(f"drift_{name}_max", mx)
        print(f"end-to-end drift {'fp8' if fp8 else 'fp16'} {name}: rms {rms:.2e} max {mx:.2e}")
        # FP16 chain: a few FP16 steps; FP8 chain: a flipped E4M3 / E5M2 code moves one product by up to 12 % of an element
        assert rms < (2e-2 if fp8 else 2e-3) and mx < (0.5 if fp8 else 2e-2), (name, rms, mx)

def _sample(n, k, seed):
    rng = np.random.default_rng(seed)
    return np.sort(rng.choice(n, size=min(k, n), replace=False))


def _variances(run):
    v = lambda name: float(torch.var(run.dev[name].float()).item())
    eh2 = float(O.gelu_scales()[0]) ** 2 * (1 / 3 + 1 / (2 * np.pi * np.sqrt(3)))
    for name in ("Z", "dZ16", "dX", "dW1"):
        assert abs(v(name) - 1.0) < 0.05, (name, v(name))
    for name in ("Y", "dW2"):
        assert abs(v(name) / eh2 - 1.0) < 0.05, (name, v(name))


def test_c2_bert_base_fp16():
    c = synth.CONFIGS["C2"]
    X, W1, W2, G = synth.ffn_inputs(c["T"], c["d"], c["f"], c["seed"])
    run = FfnRun(X, W1, W2, G, fp8=False)
    check_ffn(run, _sample(c["T"], 48, 1), _sample(c["f"], 24, 2), _sample(c["d"], 24, 3))
    check_sampled_elements(run, 1024, 11)
    _variances(run)


def test_c3_bert_large_fp8():
    c = synth.CONFIGS["C3"]
    X, W1, W2, G = synth.ffn_inputs(c["T"], c["d"], c["f"], c["seed"])
    run = FfnRun(X, W1, W2, G, fp8=True)
    check_ffn(run, _sample(c["T"], 48, 4), _sample(c["f"], 24, 5), _sample(c["d"], 24, 6))
    check_sampled_elements(run, 1024, 12)
    _variances(run)
    _same_without_fp16_dz(run, X, W1, W2, G)


def test_c5_llm_size_fp8_sampled():
    """T=32768, d=4096, f=16384: inputs drawn on the GPU.  The oracle (about 1e10 multiply-adds per second on the host)
    checks a slab of 512 consecutive tokens through the forward pass and both grad_X products (rows are independent), a
    slab of 256 rows of dW2 and of 256 columns of dW1 over all tokens (the cheaper direction of each), a few scattered
    rows of both, and 4096 uniformly drawn elements of every stored tensor."""
    c = synth.CONFIGS["C5"]
    T, d, f = c["T"], c["d"], c["f"]
    X = synth.normal_on_device(c["seed"], synth.T_X, (T, d))
    W1 = synth.normal_on_device(c["seed"], synth.T_W1, (d, f))
    W2 = synth.normal_on_device(c["seed"], synth.T_W2, (f, d))
    G = synth.normal_on_device(c["seed"], synth.T_G, (T, d))
    run = FfnRun(X, W1, W2, G, fp8=True)
    t0 = 11 * 512 + 256                      # the slab straddles two rows of large tiles
    check_ffn(run, np.arange(t0, t0 + 512), np.concatenate([np.arange(5000, 5256), _sample(f, 3, 8)]), _sample(d, 3, 9),
              dw1_cols=np.arange(9088, 9088 + 256))
    check_sampled_elements(run, 4096, 13)
    _variances(run)


def test_hip_graph_replays_match_eager():
    """The whole step (casts + FFN forward + backward) captured in a HIP graph: every replay, with
    eager work and synchronisations in between, reproduces the eager result bit for bit."""
    T, d, f = 512, 256, 1024
    X, W1, W2, G = synth.ffn_inputs(T, d, f, seed=131)
    eager = FfnRun(X, W1, W2, G, fp8=True)
    names = ("Z", "H", "Y", "dZ16", "dZ8", "dX", "dW1", "dW2")
    want = {k: eager.full(k) for k in names}
    dev = eager.dev
    wsb = us.ffn_workspace_bytes(T, d, f)
    ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device=DEV)

    def step():
        st = stream()
        for k, fmt in (("X", us.E4M3), ("W1", us.E4M3), ("W2", us.E4M3), ("G", us.E5M2)):
            us.cast_fp8(ptr(dev[k]), us.F16, ptr(dev[k + "op"]), fmt, dev[k].numel(), 1.0, None, st)
        us.ffn_fwd(ptr(dev["Xop"]), ptr(dev["W1op"]), ptr(dev["W2op"]), ptr(dev["Z"]), ptr(dev["H"]), ptr(dev["Y"]),
                   T, d, f, True, ptr(ws), wsb, st)
        us.ffn_bwd(ptr(dev["Xop"]), ptr(dev["W1op"]), ptr(dev["W2op"]), ptr(dev["Z"]), ptr(dev["H"]), ptr(dev["Gop"]),
                   ptr(dev["dZ16"]), ptr(dev["dZ8"]), ptr(dev["dX"]), ptr(dev["dW1"]), ptr(dev["dW2"]), T, d, f, True,
                   ptr(ws), wsb, st)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(4):
        for k in names:                                   # eager work between replays: wipe the outputs
            dev[k].zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k in names:
            assert np.array_equal(dev[k].cpu().numpy(), want[k]), (rep, k)


def test_a_failing_composite_call_leaves_its_outputs_untouched():
    """Every argument of every product of us_ffn_fwd / us_ffn_bwd is checked before the first launch: a bad argument that
    only the second product uses (a misaligned Y, a misaligned dW1) must not let the first product run."""
    T, d, f = 256, 128, 512
    X, W1, W2, G = synth.ffn_inputs(T, d, f, seed=139)
    tX, tW1, tW2, tG = (to_dev(a) for a in (X, W1, W2, G))
    fill = lambda shape: torch.full(shape, 7.0, dtype=torch.float16, device=DEV)
    Z, H, Y, dZ, dX, dW1, dW2 = fill((T, f)), fill((T, f)), fill((T * d + 8,)), fill((T, f)), fill((T, d)), fill((d * f + 8,)), fill((f, d))
    wsb = us.ffn_workspace_bytes(T, d, f)
    ws = torch.zeros(max(wsb, 16), dtype=torch.uint8, device=DEV)
    with pytest.raises(us.UsError) as e:
        us.ffn_fwd(ptr(tX), ptr(tW1), ptr(tW2), ptr(Z), ptr(H), ptr(Y) + 2, T, d, f, 0, ptr(ws), wsb, stream())
    assert e.value.status == 3
    with pytest.raises(us.UsError) as e:
        us.ffn_bwd(ptr(tX), ptr(tW1), ptr(tW2), ptr(Z), ptr(H), ptr(tG), ptr(dZ), None, ptr(dX), ptr(dW1) + 2, ptr(dW2), T, d, f, 0,
                   ptr(ws), wsb, stream())
    assert e.value.status == 3
    torch.cuda.synchronize()
    for t in (Z, H, Y, dZ, dX, dW1, dW2):
        assert bool((t == 7.0).all())
    assert bool((ws == 0).all())
