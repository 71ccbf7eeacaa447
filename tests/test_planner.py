"""Planner-lite (Sec. 3.4: the launch size that maximises b / c(b) within the budget; Sec. 3.3.1:
the macroblock budget of a bin batch) on hand-made cost tables - host logic only."""
import pytest

from paper_2407_16990_amd import planner as P


# c(b) = 1 ms fixed + 0.5 ms per bin up to 8 bins, then 0.25 ms per bin (a launch that fills the chip better)
HAND = [(1, 1.5), (8, 5.0), (16, 7.0), (64, 19.0)]


def test_cost_interpolates_and_extrapolates():
    assert P.cost(HAND, 0) == 0.0
    assert P.cost(HAND, 1) == 1.5 and P.cost(HAND, 8) == 5.0
    assert P.cost(HAND, 12) == pytest.approx(6.0)                 # halfway between 8 and 16
    assert P.cost(HAND, 128) == pytest.approx(19.0 + 64 * 0.25)   # along the last segment's slope
    assert P.cost([(4, 2.0)], 2) == 2.0 and P.cost([(4, 2.0)], 8) == pytest.approx(4.0)
    with pytest.raises(ValueError):
        P.cost([], 3)


def test_best_launch_size_is_the_argmax_of_b_over_c_within_the_budget():
    # rates: b=1: .667, 8: 1.6, 16: 2.29, 64: 3.37 -> unbounded: the largest allowed
    assert P.best_launch_size(HAND, 64) == 64
    assert P.best_launch_size(HAND, 10) == 10
    # a 7 ms budget admits at most 16 bins; 6 ms at most 12
    assert P.best_launch_size(HAND, 64, budget_ms=7.0) == 16
    assert P.best_launch_size(HAND, 64, budget_ms=6.0) == 12
    assert P.best_launch_size(HAND, 64, budget_ms=1.0) == 0        # nothing fits
    # a curve whose rate peaks in the middle (cache spill beyond 16 bins): the peak wins, brute force agrees
    peaked = [(1, 1.0), (16, 4.0), (32, 16.0)]
    want = max(range(1, 33), key=lambda b: (b / P.cost(peaked, b), -b))
    assert P.best_launch_size(peaked, 32) == want == 16


def test_choose_prefers_the_geometry_with_the_highest_macroblock_rate():
    curve = {128: [(1, 0.2), (8, 0.5), (64, 3.4), (128, 6.7)],    # ~0.052 ms per bin at scale
             192: [(1, 0.35), (8, 1.0), (32, 3.7), (64, 7.3)]}    # 2.25 x the pixels, ~0.114 ms per bin
    cands = [P.Candidate(128, 0, 76, 1632), P.Candidate(192, 0, 30, 1632), P.Candidate(128, 1, 182, 1632)]
    c = P.choose(curve, cands)
    # 76 bins of 128: 4.0 ms; 30 bins of 192: 3.47 ms; one box per macroblock: 182 bins, 9.5 ms
    assert (c.bin_size, c.max_box_mbs, c.launches, c.bins_per_launch) == (192, 0, 1, 30)
    assert c.ms_per_batch == pytest.approx(P.cost(curve[192], 30))
    assert c.macroblocks_per_s == pytest.approx(1632 / (c.ms_per_batch * 1e-3))
    # a 2 ms launch budget: 192-bins go 16 per launch (1.9 ms), 128-bins 36 per launch; the faster total wins
    c2 = P.choose(curve, cands, budget_ms=2.0)
    per128 = P.best_launch_size(curve[128], 76, 2.0); per192 = P.best_launch_size(curve[192], 30, 2.0)
    t128, _ = P.batch_time(curve[128], 76, per128); t192, _ = P.batch_time(curve[192], 30, per192)
    assert c2.bin_size == (128 if t128 < t192 else 192) and c2.ms_per_batch == pytest.approx(min(t128, t192))
    assert P.cost(curve[c2.bin_size], c2.bins_per_launch) <= 2.0 and c2.launches >= 2
    # the other steps' time enters the rate but not the choice between equal extras
    c3 = P.choose(curve, cands, other_ms=0.3)
    assert c3.bin_size == 192 and c3.ms_per_batch == pytest.approx(c.ms_per_batch + 0.3)
    with pytest.raises(ValueError):
        P.choose(curve, cands, budget_ms=0.1)
    with pytest.raises(KeyError):
        P.choose(curve, [P.Candidate(96, 0, 10, 100)])


def test_batch_time_splits_into_full_launches_and_a_rest():
    ms, n = P.batch_time(HAND, 20, 8)
    assert n == 3 and ms == pytest.approx(2 * 5.0 + P.cost(HAND, 4))
    assert P.batch_time(HAND, 0, 8) == (0.0, 0)


def test_tracked_curve_file_is_well_formed():
    """The curve measured on the MI355X and kept in the tree: every bin size has increasing batch
    sizes with increasing cost, and the library's own budget helper (Sec. 3.3.1) agrees with the
    macroblocks a bin batch can hold."""
    import os
    if not os.path.exists(P.CURVE_FILE):
        pytest.skip("no measured curve in the tree yet")
    curve = P.load_curve()
    assert curve
    for S, pts in curve.items():
        bs = [b for b, _ in pts]; cs = [c for _, c in pts]
        assert bs == sorted(set(bs)) and all(c > 0 for c in cs) and cs == sorted(cs), S
    import paper_2407_16990_amd as pkg
    lib = pkg.load_library()
    assert lib.rh_budget(128, 128, 76) == 76 * 64
