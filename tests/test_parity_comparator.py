"""The comparator of the GPU parity tests (tests/parity.py) on planted faults: CPU only.

The faults are planted in copies of a random "reference"; nothing here touches the GPU or the oracle."""
import numpy as np
import pytest

import parity


def _pair(rng, shape=(3, 4, 500, 64), noise=2.3e-3):
    ref = rng.standard_normal(shape) * np.sqrt(np.arange(1, shape[-2] + 1))[:, None]      # rows grow like a causal sum
    got = ref * (1.0 + noise * np.sqrt(3) * rng.uniform(-1, 1, shape))                   # rounding-like relative noise
    return got, ref


def test_clean_tensor_passes_all_three_measures(rng):
    got, ref = _pair(rng)
    whole, grp, row, _ = parity.measures(got, ref)
    assert 2.0e-3 < whole < 2.6e-3 and whole <= grp <= 3e-3 and grp <= row <= 4e-3
    parity.check("clean", got, ref, "bf16", lambda a: a)


def test_one_wrong_row_passes_the_whole_tensor_measure_but_not_the_row_measure(rng):
    got, ref = _pair(rng, shape=(4, 12, 2000, 64))
    got[2, 7, 1234] = ref[2, 7, 1233]                      # a token row that took its neighbour's values
    whole, grp, row, at = parity.measures(got, ref)
    assert whole <= parity.EXPECT["bf16"]                  # the old comparator would have let it through
    assert row > 0.5 and at == (2 * 12 + 7, 1234)
    with pytest.raises(AssertionError):
        parity.check("one wrong row", got, ref, "bf16", lambda a: a)


def test_one_bad_head_fails_the_group_measure(rng):
    got, ref = _pair(rng, shape=(4, 12, 300, 64))
    got[3, 5] *= 1.02                                      # 2 % off on one of 48 (b,h) pairs: whole tensor 2.9e-3 + ...
    whole, grp, row, _ = parity.measures(got, ref)
    assert whole <= parity.EXPECT["bf16"] and grp > parity.EXPECT["bf16"]
    with pytest.raises(AssertionError):
        parity.check("one bad head", got, ref, "bf16", lambda a: a)


def test_a_short_row_is_held_against_its_neighbours_scale(rng):
    got, ref = _pair(rng, shape=(1, 1, 200, 64))
    # a row whose terms cancelled: a hundredth of its neighbours' length, with their absolute rounding error
    err = got[0, 0, 100] - ref[0, 0, 100]
    ref[0, 0, 100] *= 0.01
    got[0, 0, 100] = ref[0, 0, 100] + err
    assert parity.measures(got, ref)[2] <= 4e-3            # (against its own norm it would read 0.2)
    # a row that must be zero and is, and one that must be zero and holds garbage of a hundredth of the local scale
    ref[0, 0, 10] = 0.0
    got[0, 0, 10] = 0.0
    assert parity.measures(got, ref)[2] <= 4e-3
    got[0, 0, 10] = 0.04 * np.sqrt(np.mean(np.sum(ref[0, 0, :64] ** 2, axis=-1)) / 64)
    assert parity.measures(got, ref)[2] > parity.ROW_BAR["bf16"]
    # an all-zero reference with a non-zero result has no scale at all
    assert parity.measures(np.ones((1, 1, 4, 8)), np.zeros((1, 1, 4, 8)))[2] == np.inf


def test_shapes_other_than_four_dimensional(rng):
    for shape in [(64,), (5, 64), (2, 3, 64), (0, 64), (2, 2, 1, 64)]:
        ref = rng.standard_normal(shape)
        whole, grp, row, _ = parity.measures(ref.copy(), ref)
        assert whole == 0.0 and grp == 0.0 and row == 0.0
    assert parity.measures(np.ones((2, 2)), np.zeros((2, 2)))[0] == np.inf
