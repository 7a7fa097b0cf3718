"""The error metric of the GPU parity tests (tests/parity.py) on hand-made cases: the floor, the FP8 allowance, and the
values that are compared by class (infinities and NaNs)."""
import numpy as np

import parity


def test_floor_and_relative_bound():
    ref = np.array([1.0, 2.0 ** -6, 2.0 ** -10, 0.0])
    # 2e-3 of the element above the floor, 2e-3 * 2^-6 below it
    ok = ref + np.array([1.9e-3, 3.0e-5, 3.0e-5, 3.0e-5])
    assert parity.errors(ok, ref)["gated"] <= parity.RTOL
    for i, step in enumerate([2.1e-3, 3.3e-5, 3.3e-5, 3.3e-5]):
        bad = ref.copy()
        bad[i] += step
        assert parity.errors(bad, ref)["gated"] > parity.RTOL, i
    assert abs(parity.errors(ref + 1e-5, ref)["rms"] - 1e-5) < 1e-12
    assert abs(parity.errors(ref * 1.001, ref)["unfloored_max"] - 1e-3) < 1e-9          # zero reference left out


def test_fp8_allowance_scale_and_per_element_allowance():
    ref = np.array([0.0, 0.5])
    got = ref + 2.2e-4
    assert parity.errors(got, ref)["gated"] > parity.RTOL
    assert parity.errors(got, ref, fp8=True)["gated"] <= parity.RTOL
    assert parity.errors(got * 100, ref * 100, fp8=True)["gated"] > parity.RTOL            # the allowance is in units of S
    assert parity.errors(got * 100, ref * 100, fp8=True, scale=100.0)["gated"] <= parity.RTOL
    assert parity.errors(ref + 1e-2, ref, allow=np.array([1e-2, 1e-2]))["gated"] < 1e-12
    assert parity.errors(ref + 1e-2, ref, tau=1.0)["gated"] > parity.RTOL


def test_infinities_and_nans_are_compared_by_class():
    inf, nan = np.inf, np.nan
    assert parity.errors(np.array([inf, -inf, nan, 1.0]), np.array([inf, -inf, nan, 1.0]))["gated"] == 0.0
    for got, ref in (([inf], [-inf]), ([nan], [1.0]), ([1.0], [nan]), ([inf], [3.0]), ([3.0], [inf])):
        assert parity.errors(np.array(got), np.array(ref))["gated"] == np.inf, (got, ref)
