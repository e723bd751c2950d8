"""The parity bar itself, on the CPU: the row-wise check must refuse what a whole-tensor norm lets through."""
import numpy as np
import pytest

from helpers import BF16_REL_L2, BF16_ROW_REL_L2, assert_rows_close, rel_l2, row_rel_l2


def noisy_pair(rows, cols, noise, seed):
    rng = np.random.default_rng(seed)
    want = rng.standard_normal((rows, cols))
    got = want * (1.0 + noise * rng.standard_normal((rows, cols)))
    return got, want


def test_one_wrong_row_among_512_passes_the_whole_tensor_norm_and_fails_the_row_check():
    got, want = noisy_pair(512, 4096, 1e-2, seed=1)       # the rounding noise a bf16 stage shows after 8 layers
    got[137] = np.random.default_rng(2).standard_normal(4096) * 0.2 + want[137]   # one row off by 20 %
    assert rel_l2(got, want) <= BF16_REL_L2               # the old bar does not see it
    with pytest.raises(AssertionError) as e:
        assert_rows_close(got, want, BF16_ROW_REL_L2, "planted")
    assert "137" in str(e.value)
    good, want = noisy_pair(512, 4096, 1e-2, seed=3)
    assert assert_rows_close(good, want) < 1.2e-2


def test_row_check_on_cache_shaped_tensors_names_layer_head_and_position():
    got, want = noisy_pair(2 * 2 * 4 * 40, 128, 3e-3, seed=4)
    got, want = got.reshape(2, 2, 4, 40, 128), want.reshape(2, 2, 4, 40, 128)
    assert row_rel_l2(got, want).shape == (2, 2, 4, 40)
    got[1, 0, 3, 17] = -want[1, 0, 3, 17]                 # a key with the wrong sign
    with pytest.raises(AssertionError) as e:
        assert_rows_close(got, want, BF16_ROW_REL_L2, "cache")
    assert "(1, 0, 3, 17)" in str(e.value)


def test_zero_rows_are_measured_against_the_mean_row_norm():
    want = np.ones((4, 8))
    want[2] = 0.0
    got = want.copy()
    got[2] = 1e-4                                          # tiny absolute error on a zero row: fine
    assert assert_rows_close(got, want) < BF16_ROW_REL_L2
    got[2] = 0.5
    with pytest.raises(AssertionError):
        assert_rows_close(got, want)
    assert assert_rows_close(np.zeros((0, 8)), np.zeros((0, 8))) == 0.0
