"""FFN chain of the oracle (CPU only): stage composition and the variances it should produce."""
import math

import numpy as np
import pytest

import oracle
import synth
from oracle import E4M3, E5M2


@pytest.mark.parametrize("fp8", [False, True])
def test_ffn_chain_variances(fp8):
    """Z, H, dH, dZ, dX, dW1 are unit-variance; Y and dW2 see H's non-zero mean:
    E[H^2] = alpha_g^2 E[gelu^2] = 1.230 (the activation breaks the zero-mean assumption, App. E.1)."""
    T, d, f = 512, 256, 1024
    X, W1, W2, G = synth.ffn_inputs(T, d, f, seed=61)
    fw = oracle.ffn_fwd(X, W1, W2, fp8)
    bw = oracle.ffn_bwd(X, W1, W2, G, fw, fp8)
    ag = float(oracle.gelu_scales()[0])
    eh2 = ag * ag * (1 / 3 + 1 / (2 * math.pi * math.sqrt(3)))
    assert abs(eh2 - 1.2302) < 1e-3
    var = lambda a: float(np.var(a.astype(np.float64)))
    for name, t in (("Z", fw["Z"]), ("H", fw["H"]), ("dH", bw["dH"]), ("dZ", bw["dZ"]), ("dX", bw["dX"]), ("dW1", bw["dW1"])):
        assert abs(var(t) - 1.0) < 0.05, (name, var(t))
    for name, t in (("Y", fw["Y"]), ("dW2", bw["dW2"])):
        assert abs(var(t) / eh2 - 1.0) < 0.05, (name, var(t))


def test_fp8_chain_only_quantises_matmul_inputs():
    T, d, f = 64, 64, 128
    X, W1, W2, G = synth.ffn_inputs(T, d, f, seed=67)
    fw = oracle.ffn_fwd(X, W1, W2, True)
    assert fw["Z"].dtype == np.float16 and fw["H"].dtype == np.float16 and fw["Y"].dtype == np.float16
    assert fw["X8"].dtype == np.uint8 and fw["H8"].dtype == np.uint8
    # H8 is the cast of the stored FP16 H, not of a higher-precision value
    assert np.array_equal(fw["H8"], oracle.cast_fp8(fw["H"], E4M3)[0])
    bw = oracle.ffn_bwd(X, W1, W2, G, fw, True)
    assert np.array_equal(bw["dZ8"], oracle.cast_fp8(bw["dZ"], E5M2)[0])
    # FP8 and FP16 chains agree to FP8 precision (relative RMS error of E4M3 rounding ~ 2.7 %)
    fw16 = oracle.ffn_fwd(X, W1, W2, False)
    rel = np.sqrt(np.mean((fw["Y"].astype(np.float64) - fw16["Y"].astype(np.float64)) ** 2))
    assert 0.005 < rel < 0.1
