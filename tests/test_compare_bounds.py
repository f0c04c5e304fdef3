"""The comparison used by the GPU parity tests must notice local damage that a whole-tensor norm hides (CPU only)."""
import numpy as np
import pytest

from util import assert_close


def _case(rows=8192, cols=64, seed=0):
    rng = np.random.default_rng(seed)
    want = rng.standard_normal((rows, cols))
    got = want + 1e-3 * rng.standard_normal((rows, cols))
    return got, want


def test_clean_output_passes():
    got, want = _case()
    assert assert_close(got, want, "bf16") < 2e-2


def test_one_bad_row_of_many_fails():
    got, want = _case()
    got[4097] = np.random.default_rng(1).standard_normal(got.shape[1])      # 1.6 % of the Frobenius norm: inside 2e-2
    with pytest.raises(AssertionError, match="row 4097|element"):
        assert_close(got, want, "bf16")


def test_one_bad_column_fails():
    got, want = _case(rows=64, cols=4096)
    got[:, 4095] = 0.0
    with pytest.raises(AssertionError, match="column 4095|element"):
        assert_close(got, want, "bf16")


def test_one_bad_element_fails():
    got, want = _case()
    got[17, 5] += 1.0
    with pytest.raises(AssertionError, match="element"):
        assert_close(got, want, "bf16")


def test_vector_and_zero_cases():
    v = np.linspace(-1, 1, 257)
    assert_close(v, v, "f32")
    assert_close(np.zeros((4, 4)), np.zeros((4, 4)), "f32")
    with pytest.raises(AssertionError):
        assert_close(v[:-1], v, "f32")
