"""The parity check itself: what it must reject (CPU)."""
import numpy as np
import pytest

from util import check_close


def _ref(seed=0, shape=(8, 32, 128), scale=0.02):
    return np.random.default_rng(seed).normal(size=shape) * scale


def test_accepts_bf16_rounding_noise():
    ref = _ref()
    got = ref * (1 + np.random.default_rng(1).uniform(-2 ** -9, 2 ** -9, size=ref.shape))
    check_close(got, ref, "bf16")


def test_rejects_one_row_ten_percent_off_although_the_global_norms_pass():
    ref = _ref()
    got = ref.copy()
    got[3, 7] *= 1.1  # one (stream, head) row of 256: global rel L2 = 0.1 / 16 < 1e-2, max|d| ~ 6e-3 < 2e-2
    d = got - ref
    assert np.max(np.abs(d)) < 2e-2 and np.linalg.norm(d) / np.linalg.norm(ref) < 1e-2
    with pytest.raises(AssertionError, match="row"):
        check_close(got, ref, "bf16")


def test_rejects_one_element_off_by_a_row_magnitude():
    ref = _ref(shape=(4, 8, 128))
    got = ref.copy()
    got[1, 2, 5] += 0.05 * np.max(np.abs(ref[1, 2]))  # row rel L2 stays below 1e-2
    d = got[1, 2] - ref[1, 2]
    assert np.linalg.norm(d) / np.linalg.norm(ref[1, 2]) < 1e-2
    with pytest.raises(AssertionError, match="elements beyond"):
        check_close(got, ref, "bf16")


def test_rejects_non_finite_and_shape_mismatch():
    ref = _ref(shape=(2, 2, 64))
    got = ref.copy()
    got[0, 0, 0] = np.nan
    with pytest.raises(AssertionError):
        check_close(got, ref, "bf16")
    with pytest.raises(AssertionError):
        check_close(ref[:1], ref, "bf16")


def test_fp32_bar_is_1e5():
    ref = _ref(shape=(2, 4, 64), scale=1.0)
    check_close(ref * (1 + 1e-6), ref, "f32")
    with pytest.raises(AssertionError):
        check_close(ref * (1 + 1e-4), ref, "f32")
