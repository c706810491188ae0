"""Pins for the oracle's sequence splice (pruned visual tokens into the prefill input)."""
import numpy as np
import pytest

from oracle import rtprune_oracle as orc


def test_hand_example():
    prefix = np.array([[1.0, 1.0], [2.0, 2.0]])
    visual = np.array([[10.0, 0.0], [13.0, 0.0], [14.0, 0.0]])       # kept tokens 0, 3, 4 of 6
    suffix = np.array([[7.0, 7.0]])
    rows, pos = orc.splice_sequence(prefix, visual, suffix, [0, 3, 4], 6, orc.POSITIONS_CONSECUTIVE)
    assert rows.tolist() == [[1, 1], [2, 2], [10, 0], [13, 0], [14, 0], [7, 7]]
    assert pos.tolist() == [0, 1, 2, 3, 4, 5]
    rows2, pos2 = orc.splice_sequence(prefix, visual, suffix, [0, 3, 4], 6, orc.POSITIONS_ORIGINAL)
    assert rows2.tolist() == rows.tolist()
    assert pos2.tolist() == [0, 1, 2, 5, 6, 8]      # 2 + {0, 3, 4}; suffix at 2 + 6


def test_nothing_pruned_gives_the_unpruned_sequence_in_both_modes():
    rng = np.random.default_rng(3)
    prefix, visual, suffix = rng.standard_normal((4, 8)), rng.standard_normal((9, 8)), rng.standard_normal((3, 8))
    a = orc.splice_sequence(prefix, visual, suffix, np.arange(9), 9, orc.POSITIONS_CONSECUTIVE)
    b = orc.splice_sequence(prefix, visual, suffix, np.arange(9), 9, orc.POSITIONS_ORIGINAL)
    np.testing.assert_array_equal(a[0], b[0])
    np.testing.assert_array_equal(a[1], b[1])
    np.testing.assert_array_equal(a[1], np.arange(16))


def test_positions_are_increasing_and_text_rows_untouched():
    rng = np.random.default_rng(4)
    for p_len, s_len in ((0, 0), (5, 0), (0, 2), (3, 7)):
        n = 20
        kept = np.sort(rng.choice(n, size=11, replace=False))
        prefix, suffix = rng.standard_normal((p_len, 6)), rng.standard_normal((s_len, 6))
        visual = rng.standard_normal((11, 6))
        for mode in (orc.POSITIONS_CONSECUTIVE, orc.POSITIONS_ORIGINAL):
            rows, pos = orc.splice_sequence(prefix, visual, suffix, kept, n, mode)
            assert rows.shape == (p_len + 11 + s_len, 6) and pos.dtype == np.int32
            assert (np.diff(pos) > 0).all()
            np.testing.assert_array_equal(rows[:p_len], prefix)
            np.testing.assert_array_equal(rows[p_len:p_len + 11], visual)
            np.testing.assert_array_equal(rows[p_len + 11:], suffix)
        _, pos = orc.splice_sequence(prefix, visual, suffix, kept, n, orc.POSITIONS_ORIGINAL)
        np.testing.assert_array_equal(pos[p_len:p_len + 11] - p_len, kept)
        assert pos[-1] <= p_len + n + s_len - 1
    with pytest.raises(ValueError):
        orc.splice_sequence(prefix, visual, suffix, kept, n, 2)
