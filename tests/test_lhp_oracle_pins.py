"""Pins of the latency-hysteresis oracle (no GPU, and nothing of the product): hand-worked curves whose hysteresis
points, redundancy and growth targets follow from the definitions of the paper's Section 3 (a hysteresis point is
where a stretch of no-faster smaller dimensions begins; redundancy = (1 - #points kept / #points) * 100 %, the
formula in the caption of the model-level latency figure) and from Section 5.1 step (c) (1197 is grown back to the
1200 the device favours).  Every expected value below is written out by hand, none comes from a program."""
import itertools

import pytest

from oracle import lhp as olhp


def test_staircase_by_hand():
    # two plateaus; 192 is a local bump above its plateau
    dims = [64, 96, 128, 160, 192, 224, 256]
    lat = [10.0, 10.0, 10.0, 20.0, 21.0, 20.0, 20.0]
    flags, red = olhp.find_lhp(dims, lat, 0.0)
    # 256: largest, always.  224, 160: equal to 256, not strictly faster.  192: slower.  128: below everything above
    # it.  96, 64: tie with 128, not strictly faster -> inside 128's stretch.
    assert flags == [0, 0, 1, 0, 0, 0, 1]
    assert red == pytest.approx((1 - 2 / 7) * 100, abs=1e-12)


def test_strictly_increasing_curve_has_no_redundancy():
    dims = [8, 16, 24, 32, 40]
    lat = [1.0, 2.0, 3.0, 4.0, 5.0]
    flags, red = olhp.find_lhp(dims, lat, 0.0)
    assert flags == [1, 1, 1, 1, 1] and red == 0.0


def test_decreasing_curve_keeps_only_the_largest():
    # every smaller dimension is slower than the largest: all of them lie in its stretch
    dims = [8, 16, 24, 32]
    lat = [4.0, 3.0, 2.0, 1.0]
    flags, red = olhp.find_lhp(dims, lat, 0.0)
    assert flags == [0, 0, 0, 1] and red == 75.0


def test_single_point_and_unsorted_input():
    assert olhp.find_lhp([100], [3.0], 0.0) == ([1], 0.0)
    # same staircase, shuffled: the flags follow the points, not the positions
    dims = [192, 64, 256, 128, 96, 224, 160]
    lat = [21.0, 10.0, 20.0, 10.0, 10.0, 20.0, 20.0]
    flags, _ = olhp.find_lhp(dims, lat, 0.0)
    assert flags == [0, 0, 1, 1, 0, 0, 0]


def test_margin_by_hand():
    # 100 -> 98.5 is a 1.5 % gain, 98.5 -> 90 a larger one
    dims = [1, 2, 3]
    lat = [90.0, 98.5, 100.0]
    assert olhp.find_lhp(dims, lat, 0.0)[0] == [1, 1, 1]
    # eps = 2 %: 98.5 is not below 0.98 * 100 = 98 -> not a point; 90 < 0.98 * 98.5 = 96.53 and < 98 -> a point
    assert olhp.find_lhp(dims, lat, 0.02)[0] == [1, 0, 1]
    # eps = 10 %: 90 is not below 0.9 * 98.5 = 88.65 -> only the largest is left
    flags, red = olhp.find_lhp(dims, lat, 0.10)
    assert flags == [0, 0, 1] and red == pytest.approx(200 / 3, abs=1e-12)


def test_a_point_is_judged_against_every_larger_dimension_not_only_the_next():
    # 3 beats its neighbour 4 but not the dip at 5
    dims = [3, 4, 5, 6]
    lat = [5.0, 9.0, 4.0, 10.0]
    assert olhp.find_lhp(dims, lat, 0.0)[0] == [0, 0, 1, 1]


def test_flags_are_exactly_the_strict_running_minimum_from_the_right():
    """For eps = 0 the definition is equivalent to: scanning from the largest dimension down, a point is kept iff it
    is strictly below the minimum seen so far.  Checked exhaustively over all curves of 5 points with 3 levels."""
    dims = [10, 20, 30, 40, 50]
    for lat in itertools.product([1.0, 2.0, 3.0], repeat=5):
        want, best = [0] * 5, float("inf")
        for i in range(4, -1, -1):
            if lat[i] < best:
                want[i] = 1
                best = lat[i]
        assert olhp.find_lhp(dims, list(lat), 0.0)[0] == want


def test_growth_target_by_hand():
    # 1197 sits on the tier of 1200 and is a shade slower than it (a stretch that begins at 1200)
    dims = [1136, 1168, 1197, 1200, 1232, 1264]
    lat = [70.0, 70.1, 75.2, 75.0, 75.1, 80.0]
    # points: 1264 (largest), 1232 (75.1 < 80), 1200 (75.0 < 75.1), not 1197 (75.2 > 75.0), 1168 (70.1), 1136 (70.0)
    assert olhp.find_lhp(dims, lat, 0.0)[0] == [1, 1, 0, 1, 1, 1]
    target, gain = olhp.grow_to_lhp(dims, lat, 1197)
    assert target == 1200 and gain == pytest.approx((1 - 75.0 / 75.2) * 100, abs=1e-12)
    assert olhp.grow_to_lhp(dims, lat, 1169)[0] == 1200        # 1169 was not measured: first measured above is 1197
    assert olhp.grow_to_lhp(dims, lat, 1168) == (1168, 0.0)    # a point that is one stays
    assert olhp.grow_to_lhp(dims, lat, 1201)[0] == 1232
    assert olhp.grow_to_lhp(dims, lat, 1264) == (1264, 0.0)
    with pytest.raises(ValueError):
        olhp.grow_to_lhp(dims, lat, 1265)


def test_growth_target_with_margin_by_hand():
    dims = [100, 104, 108, 112]
    lat = [50.0, 59.5, 60.0, 60.0]
    # eps 2 %: 112 always; 108 ties; 104: 59.5 is not below 58.8; 100: 50 < 0.98 * 59.5 -> points 100, 112
    assert olhp.find_lhp(dims, lat, 0.02)[0] == [1, 0, 0, 1]
    target, gain = olhp.grow_to_lhp(dims, lat, 101, 0.02)
    # smallest measured dimension >= 101 is 104 (59.5); the target is 112 (60.0): growing there costs 0.84 %
    assert target == 112 and gain == pytest.approx((1 - 60.0 / 59.5) * 100, abs=1e-12)
    assert olhp.grow_to_lhp(dims, lat, 100, 0.02) == (100, 0.0)
