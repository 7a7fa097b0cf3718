"""The Gaussian-tail coefficients compiled into the kernels (csrc/us_device.h, gauss_terms) against their generator and
against scipy's scaled complementary error function: the constants must be the ones the committed fit produces (to the
flatness of its minimum) and keep the relative accuracy the header states."""
import importlib.util
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
PATH = os.path.join(os.path.dirname(HERE), "paper_2303_11257_amd", "csrc", "fit_gauss_tail.py")


def _generator():
    spec = importlib.util.spec_from_file_location("fit_gauss_tail", PATH)
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_compiled_constants_keep_their_stated_accuracy():
    g = _generator()
    p, cs = g.compiled_constants()
    assert g.max_relative_error(p, cs) < 4.0e-6                       # exact arithmetic: the header's bound
    assert g.max_relative_error(p, cs, np.float32) < 5.0e-6           # the kernel's FP32 Horner evaluation


def test_a_fresh_fit_lands_on_the_compiled_constants():
    g = _generator()
    p, cs = g.compiled_constants()
    c, err = g.fit(p, 200)                                            # same p: the coefficients are then determined
    assert err < 4.0e-6
    assert np.max(np.abs(c - np.array(cs))) < 5e-5
