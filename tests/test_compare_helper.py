"""The comparison the GPU parity tests use must be able to fail on a local error: planted on the
CPU, in a copy of an oracle-sized tensor (no GPU involved)."""
import numpy as np
import pytest

from _gpu_util import assert_matches, rel_fro


def _tensor(rows=16384, cols=96, seed=3):
    return np.random.default_rng(seed).standard_normal((rows, cols))


def test_equal_tensors_and_rounding_noise_pass():
    want = _tensor()
    assert assert_matches(want.copy(), want, 2e-2) == 0.0
    noisy = want * (1 + 2.0 ** -9 * np.random.default_rng(4).uniform(-1, 1, want.shape))
    assert assert_matches(noisy, want, 2e-2) < 3e-3


def test_one_wrong_row_among_many_fails_although_the_norm_passes():
    want = _tensor()
    got = want.copy()
    got[777] = 0.0                       # a token row that was never computed
    assert rel_fro(got, want) < 2e-2     # the whole-tensor norm does not see it
    with pytest.raises(AssertionError, match="rows beyond the bound"):
        assert_matches(got, want, 2e-2)


def test_one_wrong_element_fails():
    want = _tensor()
    got = want.copy()
    got[5, 7] += 1.0
    assert rel_fro(got, want) < 2e-2
    with pytest.raises(AssertionError):
        assert_matches(got, want, 2e-2)


def test_a_nan_fails():
    want = _tensor(64, 8)
    got = want.copy()
    got[3, 3] = np.nan
    with pytest.raises(AssertionError, match="non-finite"):
        assert_matches(got, want, 2e-2)


def test_small_rows_are_held_to_the_typical_row_norm_not_their_own():
    # a row that is nearly zero in the oracle may carry rounding noise of the typical magnitude
    want = _tensor(256, 32)
    want[10] *= 1e-6
    got = want.copy()
    got[10] += 1e-3 * np.random.default_rng(5).standard_normal(32)
    assert_matches(got, want, 2e-2)
