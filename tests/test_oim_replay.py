"""CPU checks of the acceptance rule for OIM maps at decisions the arithmetic cannot resolve (tests/oim_replay.py):
it must reproduce the oracle where the GPU agrees with it, follow an alternative that is within the tolerance, and
refuse to follow one that is not (the planted mistakes live here, on the CPU)."""
import numpy as np
import pytest

from oim_replay import replay

W_AX, H_AX = 1, 0


@pytest.mark.parametrize("R", [1, 0, 2])
@pytest.mark.parametrize("passes", [[(W_AX, 3)], [(H_AX, 2), (W_AX, 4)], [(W_AX, 2), (H_AX, 2), (W_AX, 2), (H_AX, 1)]])
def test_replay_of_the_oracles_own_maps_is_the_oracle(oracle, passes, R):
    rng = np.random.default_rng(50 + R)
    x = rng.standard_normal((2, 6, 9, 5))
    s = rng.integers(1, 4, (2, 6, 9))
    for rm in (oracle.ROUND_NONE, oracle.ROUND_BF16):
        ref = oracle.oim_merge(x, passes, sizes=s, R=R, round_mode=rm)
        got = replay(oracle, x, passes, ref["merged_map"], sizes=s, R=R, round_mode=rm)
        for k in ("x", "sizes", "merged_map", "kept_map"):
            np.testing.assert_array_equal(got[k], ref[k])
        assert got["close"] == 0
        # a map that has nothing to do with the input changes nothing while every decision is clear
        junk = rng.integers(0, ref["x"].shape[1] * ref["x"].shape[2], ref["merged_map"].shape).astype(np.int32)
        got = replay(oracle, x, passes, junk, sizes=s, R=R, round_mode=rm)
        np.testing.assert_array_equal(got["merged_map"], ref["merged_map"])


def test_replay_keyed(oracle):
    rng = np.random.default_rng(53)
    x, keys = rng.standard_normal((2, 5, 8, 4)), rng.standard_normal((2, 5, 8, 6))
    passes = [(W_AX, 3), (H_AX, 2)]
    ref = oracle.oim_merge_keyed(x, keys, passes, round_mode=oracle.ROUND_BF16)
    got = replay(oracle, x, passes, ref["merged_map"], round_mode=oracle.ROUND_BF16, metric=keys)
    for k in ("x", "metric", "sizes", "merged_map", "kept_map"):
        np.testing.assert_array_equal(got[k], ref[k])


def test_an_alternative_within_the_tolerance_is_followed_and_one_outside_is_not(oracle):
    d1 = np.array([1.0, 2.0, 3.0, -1.0])
    s2 = np.array([0.5, 2.5, 2.0, 0.0])
    far = np.array([-1.0, 0.0, 1.0, 4.0])
    # source 2 sits between destination 1 and a scaled copy of it: the two cosines agree to the last bit or two
    line = np.array([d1, d1, s2, 3.0 * d1, far]).reshape(1, 1, 5, 4)
    passes = [(W_AX, 3)]
    ref = oracle.oim_merge(line, passes)
    assert ref["margin"] < 1e-14
    to_left, to_right = np.array([[0, 0, 0, 1, 1]], np.int32), np.array([[0, 0, 1, 1, 1]], np.int32)
    for alt in (to_left, to_right):
        got = replay(oracle, line, passes, alt)
        np.testing.assert_array_equal(got["merged_map"], alt)
        assert got["close"] == 1
    np.testing.assert_allclose(replay(oracle, line, passes, to_right)["x"][0, 0], [(d1 + d1) / 2, (3 * d1 + s2 + far) / 3], rtol=1e-15)
    np.testing.assert_array_equal(replay(oracle, line, passes, to_right)["sizes"], [[[2, 3]]])
    # a clear preference (gap 0.2 in cosine) is not given up, whatever the map under test says
    e1, e2 = np.array([1.0, 0.0, 0.0, 0.0]), np.array([0.0, 1.0, 0.0, 0.0])
    clear = np.array([e1, e1, [3.0, 4.0, 0.0, 0.0], e2, e2]).reshape(1, 1, 5, 4)
    got = replay(oracle, clear, passes, to_left)
    np.testing.assert_array_equal(got["merged_map"], to_right)
    assert got["close"] == 0


def test_a_selection_within_the_tolerance_is_followed(oracle):
    # two sources with the same score up to rounding compete for the one merge of the line
    d = np.array([2.0, 1.0, 0.0])
    a = np.array([1.0, 1.0, 1.0])
    line = np.array([a, d, 5.0 * d, 7.0 * d, 3.0 * a]).reshape(1, 1, 5, 3)      # sources 0, 2, 4; 2 is clearly the best
    ref = oracle.oim_merge(line, [(W_AX, 2)])                                     # 2 and one of {0, 4}
    first, last = np.array([[0, 0, 0, 1, 2]], np.int32), np.array([[0, 1, 1, 2, 2]], np.int32)
    assert ref["margin"] < 1e-14
    for alt in (first, last):
        got = replay(oracle, line, [(W_AX, 2)], alt)
        assert got["close"] >= 1
        assert set(np.nonzero(np.bincount(got["merged_map"][0]) > 1)[0]) == set(np.nonzero(np.bincount(alt[0]) > 1)[0])
