"""The benchmark's step launched back to back, as bench.py launches it: casts, us_ffn_fwd, us_ffn_bwd, again and again
on the same buffers with no host synchronisation in between, the inputs alternating between two seeded sets.

Every launch reads what the launch before it wrote (the E4M3 / E5M2 codes of the cast, H8, Z16, dZ8), all of it stored
write-through, and the epilogues touch cache lines of Z16 ahead of their use: an output that one launch takes from a
stale cache line, or from the other input set's step, differs from the same step run alone and synchronised.  The
references are the library's own outputs of each set, run once with a synchronisation after every call (those are compared
with the oracle in test_gpu_ffn.py); here every tensor of every repetition must equal them bit for bit."""
import pytest
import torch

import paper_2303_11257_amd as us
import synth
from gpu_util import DEV, ptr, stream, to_dev

pytestmark = pytest.mark.gpu

OUTS = ("Z", "H", "Y", "dZ", "dX", "dW1", "dW2")


class _Step:
    def __init__(self, T, d, f, fp8):
        self.T, self.d, self.f, self.fp8 = T, d, f, fp8
        e = lambda shape, dt=torch.float16: torch.empty(shape, dtype=dt, device=DEV)
        code = torch.uint8 if fp8 else torch.float16
        self.op = dict(X=e((T, d), code), W1=e((d, f), code), W2=e((f, d), code), G=e((T, d), code))
        self.out = dict(Z=e((T, f)), H=e((T, f), code), Y=e((T, d)), dZ=e((T, f), code), dX=e((T, d)), dW1=e((d, f)), dW2=e((f, d)))
        self.wsb = us.ffn_workspace_bytes(T, d, f)
        self.ws = torch.zeros(max(self.wsb, 16), dtype=torch.uint8, device=DEV)
        us.gelu_tables(ptr(self.ws), self.wsb, 0.0, 0.0, stream())
        self.mode = (us.FFN_FP8 if fp8 else 0) | us.FFN_TABLES_READY

    def run(self, src, sync):
        """One step on the FP16 inputs `src`; sync: wait for the device after every call."""
        st, o, op = stream(), self.out, self.op
        T, d, f = self.T, self.d, self.f
        wait = torch.cuda.synchronize if sync else (lambda: None)
        if self.fp8:
            names = ("X", "W1", "W2", "G")
            us.cast_fp8_batch([ptr(src[k]) for k in names], [ptr(op[k]) for k in names], [src[k].numel() for k in names],
                              [us.E4M3, us.E4M3, us.E4M3, us.E5M2], st)
            wait()
            x = op
        else:
            x = src
        us.ffn_fwd(ptr(x["X"]), ptr(x["W1"]), ptr(x["W2"]), ptr(o["Z"]), ptr(o["H"]), ptr(o["Y"]), T, d, f, self.mode,
                   ptr(self.ws), self.wsb, st)
        wait()
        us.ffn_bwd(ptr(x["X"]), ptr(x["W1"]), ptr(x["W2"]), ptr(o["Z"]), ptr(o["H"]), ptr(x["G"]),
                   None if self.fp8 else ptr(o["dZ"]), ptr(o["dZ"]) if self.fp8 else None, ptr(o["dX"]), ptr(o["dW1"]), ptr(o["dW2"]),
                   T, d, f, self.mode, ptr(self.ws), self.wsb, st)
        wait()


@pytest.mark.parametrize("T,d,f,fp8", [(8192, 1024, 4096, True), (4096, 768, 3072, False)], ids=["bert_large_fp8", "bert_base_fp16"])
def test_steps_back_to_back_equal_the_step_run_alone(T, d, f, fp8):
    step = _Step(T, d, f, fp8)
    sets = []
    for seed in (synth.BASE_SEED + 40, synth.BASE_SEED + 41):
        X, W1, W2, G = synth.ffn_inputs(T, d, f, seed)
        sets.append(dict(X=to_dev(X), W1=to_dev(W1), W2=to_dev(W2), G=to_dev(G)))
    refs = []
    for src in sets:
        step.run(src, sync=True)
        refs.append({k: step.out[k].clone() for k in OUTS})
    assert not torch.equal(refs[0]["Y"], refs[1]["Y"])                  # the two sets really differ
    # 24 repetitions, alternating sets, nothing but the comparisons (device-side, same stream) between the steps
    bad = torch.zeros(len(OUTS), dtype=torch.int32, device=DEV)
    for it in range(24):
        which = it & 1
        step.run(sets[which], sync=False)
        for i, k in enumerate(OUTS):
            a, b = step.out[k], refs[which][k]
            # bit patterns, so that NaNs would compare equal to themselves
            a, b = (a, b) if a.dtype == torch.uint8 else (a.view(torch.int16), b.view(torch.int16))
            bad[i] += (a != b).any().to(torch.int32)
    torch.cuda.synchronize()
    counts = dict(zip(OUTS, bad.cpu().tolist()))
    assert all(v == 0 for v in counts.values()), f"repetitions (of 24) in which a tensor differed from the step run alone: {counts}"
