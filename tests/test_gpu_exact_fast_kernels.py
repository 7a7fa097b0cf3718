"""GPU parity, bit for bit, on the kernels the benchmark workloads run (direct-to-LDS loads: 256 x 256, 256 x 128 with two
wave groups, 128 x 128 with two wave groups, plain 128 x 128, K slices, and every kind of paired backward launch).

Operands are small integers (exact in FP16 / E4M3 / E5M2) and the scales powers of two, so every partial sum is exact in
FP32 whatever the order of the additions: the GPU must equal the oracle exactly, for FP32 and FP16 outputs.  A k-step that
is dropped, added twice or taken from the wrong ring slot, a wave group's half that lands in the wrong sum, a swizzle or a
transposing read that picks the wrong element: each changes an integer.  Every case first checks, through
us_last_launch(), that the shape really runs the kernel it was chosen for.  Large outputs are compared on a strided set of
rows that meets every row of tiles (the oracle does about 1e10 multiply-adds per second)."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2303_11257_amd as us
import synth
from gpu_util import DEV, cast_fp8, empty, ptr, stream, to_dev

pytestmark = pytest.mark.gpu

# (b, m, n), and what each product of the layer must run on with FP16 results:  fwd, grad_X alone, grad_W alone, both in
# one call.  Entries are substrings of us_last_launch(); None = do not care; a dict picks by precision.  (FP32 results
# are compared too; they take the plain 128 x 128 tile wherever the FP16 result takes a wave-group tile.)
CASES = [
    # forward 192 large tiles, one stage pair of reduction; grad_X few small tiles with two wave groups; grad_W K slices
    # (FP16: the 4096 x 3072 output on 16 x 16 tiles of 256 x 192, one per CU, instead of 192 of 256 x 256)
    dict(shape=(4096, 256, 3072), fwd={"fp8": "direct:256x256:wk1", "f16": "direct:256x192:wk1:st2:f16:NN"}, dx="direct:128x128:wk2:st4",
         dw="direct:128x128:wk1:st2:{p}:TN:partial:f32:s8",
         both=None),
    # forward: 256 tiles of 256 x 128 (FP8) / plain small tiles (FP16); backward pair: wave-split small grad_X + long grad_W tiles
    dict(shape=(2048, 1024, 4096), fwd={"fp8": "direct:256x128:wk2:st3", "f16": "direct:128x128:wk1:st2"}, dx="direct:128x128:wk2:st4",
         dw="direct:128x128:wk2:st2:{p}:TN", both="pair:128x128:wk2:st4:{p}:NT:store:s1 + pair:256x128:wk2:st3:{p}:TN"),
    # the BERT-large layer-2 backward shape with fewer tokens: large grad_X tiles + long grad_W tiles in one launch
    dict(shape=(6144, 4096, 1024), fwd={"fp8": "direct:256x128:wk2:st3", "f16": "direct:128x128:wk1:st2"},
         dx="direct:256x256:wk1:st2:{p}:NT", dw="direct:128x128:wk2:st2:{p}:TN",
         both="pair:256x256:wk1:st2:{p}:NT:store:s1 + pair:256x128:wk2:st3:{p}:TN", stride=13),
    # the BERT-large layer-1 backward shape: one round of 128 large grad_X tiles + 128 long grad_W tiles
    dict(shape=(8192, 1024, 4096), fwd="direct:256x256:wk1", dx={"fp8": "direct:256x128:wk2:st3", "f16": "direct:128x128:wk1:st2"},
         dw="direct:128x128:wk2:st2:{p}:TN", both="pair:256x256:wk1:st2:{p}:NT:store:s1 + pair:256x128:wk2:st3:{p}:TN", stride=17),
    # grad_X on 192 tiles of 256 x 128 next to a wave-split grad_W of 192 small tiles
    dict(shape=(3072, 2048, 1536), fwd="direct:128x128:wk1:st2", dx={"fp8": "direct:256x128:wk2:st3", "f16": "direct:128x128:wk1:st2"},
         dw="direct:128x128:wk2:st2:{p}:TN", both="pair:256x128:wk2:st3:{p}:NT:store:s1 + pair:128x128:wk2:st2:{p}:TN", stride=5),
    # the BERT-base layer-1 backward shape: grad_X on 96 tiles of 256 x 128 + grad_W on 144 wave-split small tiles, one round
    dict(shape=(4096, 768, 3072), fwd={"fp8": "direct:256x256:wk1", "f16": "direct:256x192:wk1:st2:f16:NN"}, dx="direct:128x128:wk2:st4", dw="direct:128x128:wk2:st2:{p}:TN",
         both="pair:256x128:wk2:st3:{p}:NT:store:s1 + pair:128x128:wk2:st2:{p}:TN", stride=11),
    # both on 128 x 128 tiles with two wave groups
    dict(shape=(1024, 2048, 1536), fwd="direct:128x128:wk2:st4", dx="direct:128x128:wk2:st4", dw="direct:128x128:wk2:st2:{p}:TN",
         both="pair:128x128:wk2:st4:{p}:NT:store:s1 + pair:128x128:wk2:st2:{p}:TN"),
    # grad_W on the large tile (192 tiles)
    dict(shape=(512, 4096, 3072), fwd="direct:128x128:wk2:st4", dx="direct:128x128:wk2:st4", dw="direct:256x256:wk1:st2:{p}:TN", both=None,
         stride=7),
]


def _want(entry, fp8):
    if entry is None:
        return None
    if isinstance(entry, dict):
        entry = entry["fp8" if fp8 else "f16"]
    return entry.replace("{p}", "fp8" if fp8 else "f16")


def _launched(want, what):
    got = us.last_launch()
    if want is not None:
        assert want in got, f"{what}: expected a launch like '{want}', the library chose '{got}'"
    return got


class _Layer:
    """Device operands of one linear layer with integer entries; products through the C ABI."""

    def __init__(self, b, m, n, fp8, seed):
        self.b, self.m, self.n, self.fp8 = b, m, n, fp8
        X, W, G = (synth.small_ints(seed, t, s) for t, s in ((1, (b, m)), (2, (m, n)), (4, (b, n))))
        if fp8:
            X, W, G = cast_fp8(X, us.E4M3), cast_fp8(W, us.E4M3), cast_fp8(G, us.E5M2)
            self.gdt, self.odt = (us.E4M3, us.E4M3, us.E5M2), (O.E4M3, O.E4M3, O.E5M2)
        else:
            self.gdt, self.odt = (us.F16,) * 3, (O.F16,) * 3
        self.X, self.W, self.G = X, W, G
        self.tX, self.tW, self.tG = to_dev(X), to_dev(W), to_dev(G)
        self.wsb = us.workspace_bytes(b, m, n)
        self.ws = torch.empty(max(self.wsb, 16), dtype=torch.uint8, device=DEV)

    def fwd(self, alpha, out_dt, epi=us.EPI_NONE, aux16=None, aux8=None, workspace=False):
        Y = empty((self.b, self.n), np.float16 if out_dt == us.F16 else np.float32)
        us.linear_fwd(ptr(self.tX), ptr(self.tW), ptr(Y), self.b, self.m, self.n, self.gdt[0], self.gdt[1], out_dt, alpha, epi, 0.0,
                      ptr(aux16), ptr(aux8), ptr(self.ws) if workspace else None, self.wsb if workspace else 0, stream())
        return Y

    def bwd(self, bx, bw, out_dt, dx=True, dw=True, epi=us.EPI_NONE, epi_scale=0.0, Zpre=None, aux8=None):
        odt = np.float16 if out_dt == us.F16 else np.float32
        dX = empty((self.b, self.m), odt) if dx else None
        dW = empty((self.m, self.n), odt) if dw else None
        us.linear_bwd(ptr(self.tX) if dw else None, ptr(self.tW) if dx else None, ptr(self.tG), ptr(dX), ptr(dW), self.b, self.m,
                      self.n, *self.gdt, out_dt, bx, bw, epi, epi_scale, ptr(Zpre), ptr(aux8), ptr(self.ws), self.wsb, stream())
        return dX, dW


def _rows(extent, stride):
    r = np.arange(0, extent, stride)
    return np.unique(np.concatenate([r, [extent - 1]]))


def _take(t, rows):
    torch.cuda.synchronize()
    return t[torch.as_tensor(rows, device=DEV)].cpu().numpy()


@pytest.mark.parametrize("fp8", [False, True])
@pytest.mark.parametrize("case", CASES, ids=lambda c: "x".join(map(str, c["shape"])))
def test_integer_operands_on_the_fast_kernels(case, fp8):
    b, m, n = case["shape"]
    stride = case.get("stride", 1)
    L = _Layer(b, m, n, fp8, 211 + b + m)
    X, W, G, (ox, ow, og) = L.X, L.W, L.G, L.odt
    rb, rm = _rows(b, stride), _rows(m, stride)
    alpha, bx, bw = 2.0 ** -4, 2.0 ** -5, 2.0 ** -6
    # the oracle once per product in FP32; an exact value times a power of two rounds to FP16 in one way only, which the
    # oracle's own FP16 output confirms on the forward product
    Yref = O.linear_fwd(X[rb], W, alpha, ox, ow, O.F32)
    dXref = O.linear_bwd_dx(G[rb], W, bx, og, ow, O.F32)
    dWref = O.linear_bwd_dw(np.ascontiguousarray(X[:, rm]), G, bw, ox, og, O.F32)
    assert np.array_equal(O.linear_fwd(X[rb[:8]], W, alpha, ox, ow, O.F16), Yref[:8].astype(np.float16))
    for out_g in (us.F32, us.F16):
        cast = (lambda a: a) if out_g == us.F32 else (lambda a: a.astype(np.float16))
        want = (lambda key: _want(case[key], fp8)) if out_g == us.F16 else (lambda key: None)
        Y = L.fwd(alpha, out_g)
        rec = _launched(want("fwd"), "forward")
        assert np.array_equal(_take(Y, rb), cast(Yref)), f"forward ({rec})"
        dX, _ = L.bwd(bx, bw, out_g, dw=False)
        rec = _launched(want("dx"), "grad_X alone")
        assert np.array_equal(_take(dX, rb), cast(dXref)), f"grad_X ({rec})"
        _, dW = L.bwd(bx, bw, out_g, dx=False)
        rec = _launched(want("dw"), "grad_W alone")
        assert np.array_equal(_take(dW, rm), cast(dWref)), f"grad_W ({rec})"
    # both in one call (one launch where the shapes pair up; FP16 results)
    dX, dW = L.bwd(bx, bw, us.F16)
    rec = _launched(_want(case["both"], fp8), "grad_X and grad_W in one call")
    assert np.array_equal(_take(dX, rb), dXref.astype(np.float16)), f"grad_X in one call ({rec})"
    assert np.array_equal(_take(dW, rm), dWref.astype(np.float16)), f"grad_W in one call ({rec})"


@pytest.mark.parametrize("fp8", [False, True])
@pytest.mark.parametrize("fshape,shape,both", [
    ((4096, 256, 3072), (6144, 4096, 1024), "pair:256x256:wk1:st2:{p}:NT:gelu_grad_tab:s1 + pair:256x128:wk2:st3:{p}:TN"),
    (None, (3072, 2048, 1536), "pair:256x128:wk2:st3:{p}:NT:act_grad:s1 + pair:128x128:wk2:st2:{p}:TN"),
    # the BERT-base layer-2 backward shape: grad_X on 384 tiles of 128 x 256 next to 144 grad_W tiles
    (None, (4096, 3072, 768), "pair:128x256:wk1:st2:{p}:NT:gelu_grad_tab:s1 + pair:128x128:wk2:st2:{p}:TN"),
])
def test_integer_operands_through_the_fused_epilogues(fshape, shape, both, fp8):
    """The activation epilogues on the same exact products.  Forward: the stored pre-activation Z must be the exact
    product (the activation output is compared elsewhere: it is not an integer).  Backward: with an activation scale of
    one and a pre-activation of +-9 everywhere, gelu' is exactly 1 (z = 9) or 0 (z = -9) in FP32 and in the oracle's
    double arithmetic, so dZ is the exact product where z > 0 and zero elsewhere: the sign pattern is index-coded,
    which pins the addressing of the saved pre-activation in the table-driven and the arithmetic epilogue."""
    alpha, bx, bw = 2.0 ** -4, 2.0 ** -5, 2.0 ** -6
    p = "fp8" if fp8 else "f16"
    if fshape is not None:        # forward with the table-driven GELU on the large tile
        b, m, n = fshape
        F = _Layer(b, m, n, fp8, 227 + b)
        rf = _rows(b, 11)
        H16 = empty((b, n), np.float16) if not fp8 else None
        H8 = empty((b, n), np.uint8) if fp8 else None
        Z = F.fwd(alpha, us.F16, epi=us.EPI_GELU, aux16=H16, aux8=H8, workspace=True)
        rec = _launched(f"direct:{'256x256' if fp8 else '256x192'}:wk1:st2:{p}:NN:gelu_tab", "forward with GELU")
        assert np.array_equal(_take(Z, rf), O.linear_fwd(F.X[rf], F.W, alpha, F.odt[0], F.odt[1], O.F16)), f"Z ({rec})"
        del F, Z, H16, H8
    b, m, n = shape
    L = _Layer(b, m, n, fp8, 223 + b)
    X, W, G, (ox, ow, og) = L.X, L.W, L.G, L.odt
    rb, rm = _rows(b, 11), _rows(m, 11)
    i, k = np.meshgrid(np.arange(b), np.arange(m), indexing="ij")
    sign = np.where((3 * i + 5 * k) % 7 < 3, 1.0, -1.0)
    Zpre = (9.0 * sign).astype(np.float16)
    tZ = to_dev(Zpre)
    dZ8 = empty((b, m), np.uint8) if fp8 else None
    dZ, dW = L.bwd(bx, bw, us.F16, epi=us.EPI_GELU_GRAD, epi_scale=1.0, Zpre=tZ, aux8=dZ8)
    rec = _launched(_want(both, fp8), "backward with the activation derivative")
    dH = O.linear_bwd_dx(G[rb], W, bx, og, ow, O.F16)
    ref = O.gelu_bwd(Zpre[rb], dH, 1.0)
    assert np.array_equal(ref, np.where(sign[rb] > 0, dH, np.float16(0)))          # the oracle agrees that this case is exact
    got = _take(dZ, rb)
    assert np.array_equal(got, ref), f"dZ ({rec})"
    if fp8:
        assert np.array_equal(_take(dZ8, rb), O.cast_fp8(got, O.E5M2)[0])
    assert np.array_equal(_take(dW, rm), O.linear_bwd_dw(np.ascontiguousarray(X[:, rm]), G, bw, ox, og, O.F16)), f"dW ({rec})"


@pytest.mark.parametrize("fp8", [False, True])
def test_permutation_operands_per_layout(fp8):
    """One operand is a permutation matrix, the other index-coded: the result is a permuted copy, so a transposed or
    shifted index in any of the three operand layouts (forward: weights K-strided; grad_X: both K-contiguous; grad_W:
    both K-strided) shows as a wrong element.  1024 in every dimension: direct-to-LDS kernels with two wave groups."""
    N = 1024
    i, k = np.meshgrid(np.arange(N), np.arange(N), indexing="ij")
    A = (((i + 2 * k) % 5) - 2).astype(np.float16)               # A[i, k] = (i + 2k) mod 5 - 2, not symmetric
    perm = (np.arange(N) * 7 + 3) % N
    P = np.zeros((N, N), np.float16)
    P[np.arange(N), perm] = 1.0                                   # P[k, perm[k]] = 1
    if fp8:
        enc = lambda a, f: cast_fp8(a, f)
        gdt = (us.E4M3, us.E4M3, us.E5M2)
    else:
        enc = lambda a, f: a
        gdt = (us.F16,) * 3
    st = stream()
    out = empty((N, N), np.float32)
    ws = torch.empty(us.workspace_bytes(N, N, N), dtype=torch.uint8, device=DEV)
    A32 = A.astype(np.float32)
    # forward: Y = X P  ->  Y[:, perm[k]] = X[:, k]
    tX, tW = to_dev(enc(A, us.E4M3)), to_dev(enc(P, us.E4M3))
    us.linear_fwd(ptr(tX), ptr(tW), ptr(out), N, N, N, gdt[0], gdt[1], us.F32, 1.0, us.EPI_NONE, 0.0, None, None, None, 0, st)
    assert "direct" in us.last_launch()
    Y = out.cpu().numpy()
    assert np.array_equal(Y[:, perm], A32)
    # grad_X: dX = G P^T  ->  dX[:, k] = G[:, perm[k]]
    tG = to_dev(enc(A, us.E5M2))
    us.linear_bwd(None, ptr(tW), ptr(tG), ptr(out), None, N, N, N, *gdt, us.F32, 1.0, 1.0, us.EPI_NONE, 0.0, None, None, ptr(ws), ws.numel(), st)
    assert "direct" in us.last_launch() and ":NT:" in us.last_launch()
    assert np.array_equal(out.cpu().numpy(), A32[:, perm])
    # grad_W: dW = P^T G (X = P: token t is one-hot at perm[t])  ->  dW[perm[t], :] = G[t, :]
    us.linear_bwd(ptr(tW), None, ptr(tG), None, ptr(out), N, N, N, *gdt, us.F32, 1.0, 1.0, us.EPI_NONE, 0.0, None, None, ptr(ws), ws.numel(), st)
    assert "direct" in us.last_launch() and ":TN:" in us.last_launch()
    assert np.array_equal(out.cpu().numpy()[perm], A32)
    # ... and with the index-coded matrix as the left operand of grad_W: dW = A^T P  ->  dW[:, perm[t]] = A[t, :]
    tXa, tGp = to_dev(enc(A, us.E4M3)), to_dev(enc(P, us.E5M2))
    us.linear_bwd(ptr(tXa), None, ptr(tGp), None, ptr(out), N, N, N, *gdt, us.F32, 1.0, 1.0, us.EPI_NONE, 0.0, None, None, ptr(ws), ws.numel(), st)
    assert np.array_equal(out.cpu().numpy()[:, perm], A32.T)
