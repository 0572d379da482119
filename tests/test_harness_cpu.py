"""The comparison helpers of the GPU parity tests, checked on numbers worked by hand (no GPU)."""
import numpy as np
import pytest

from tests import stage_harness as H


def test_value_errors_figures():
    b = np.array([3.0, -4.0, 0.0, 0.0])             # rms = 2.5
    a = b + np.array([0.03, 0.0, 0.05, -0.01])
    e = H.value_errors(a, b)
    assert e["rms"] == pytest.approx(2.5)
    # ratios: 0.03/3 = 0.01, 0, 0.05/2.5 = 0.02, 0.01/2.5 = 0.004
    assert e["entry_max"] == pytest.approx(0.02)
    assert e["frac_above_1e-2"] == pytest.approx(0.25)
    assert e["norm_rel"] == pytest.approx(np.sqrt(0.03 ** 2 + 0.05 ** 2 + 0.01 ** 2) / 5.0)


def test_assert_values_close_is_entry_wise_at_1e_2():
    b = np.array([1.0, -2.0, 0.5, 4.0])
    ok = b * (1 + 0.009)
    H.assert_values_close(ok, b, "fine")
    bad = b.copy()
    bad[0] += 0.03                                  # rms(b) = 2.3: 0.03 / 2.3 > 1e-2
    with pytest.raises(AssertionError):
        H.assert_values_close(bad, b, "one entry off")
    H.assert_values_close(bad, b, "deep", **H.DEEP)  # inside the full-depth bound
    with pytest.raises(AssertionError):
        H.assert_values_close(b + 0.2, b, "deep, far off", **H.DEEP)
