"""Pins for the oracle's macroblock selection (Sec. 3.3.1) against brute force."""
import numpy as np
import pytest

import workloads as wl


def rank_bruteforce(imp, g0, g1):
    """O(n^2): rank of each MB = number of MBs of the segment that precede it in the
    queue (more important, or equally important with a lower flat index)."""
    v = imp.ravel()[g0:g1].astype(np.float64)
    n = len(v)
    isnan = np.isnan(v)
    ranks = np.zeros(n, dtype=np.int64)
    for i in range(n):
        for j in range(n):
            if i == j:
                continue
            if isnan[j]:
                ahead = isnan[i] and j < i
            elif isnan[i]:
                ahead = True
            else:
                ahead = v[j] > v[i] or (v[j] == v[i] and j < i)
            ranks[i] += ahead
    return ranks


@pytest.mark.parametrize("levels", [0, 10, 2])
@pytest.mark.parametrize("k", [0, 1, 7, 60, 239, 240, 1000])
def test_topk_matches_rank_definition(orc, levels, k):
    cfg = wl.replace(wl.config(1), quantize_levels=levels)
    imp = wl.make_importance(cfg)
    mask, lst = orc.select(imp, np.array([[0, 1, k]], dtype=np.uint32))
    ranks = rank_bruteforce(imp, 0, imp.size)
    want = ranks < min(k, imp.size)
    assert np.array_equal(mask.ravel().astype(bool), want)
    assert np.array_equal(lst, np.flatnonzero(want))
    assert len(lst) == min(k, imp.size)


def test_topk_specials_nan_negzero_inf(orc):
    imp = np.array([[[np.nan, -0.0, 0.0, -np.inf, np.inf, 1.0, -1.0, np.nan, 0.0]]], dtype=np.float32)
    # queue: inf(4), 1.0(5), -0(1), 0(2), 0(8), -1(6), -inf(3), nan(0), nan(7)
    order = [4, 5, 1, 2, 8, 6, 3, 0, 7]
    for k in range(10):
        mask, lst = orc.select(imp, np.array([[0, 1, k]], dtype=np.uint32))
        assert sorted(order[:k]) == lst.tolist()
    ranks = rank_bruteforce(imp, 0, 9)
    assert [int(np.flatnonzero(ranks == r)[0]) for r in range(9)] == order


def test_topk_per_segment_and_uncovered_frames(orc):
    rng = np.random.default_rng(3)
    imp = rng.random((5, 4, 6)).astype(np.float32)
    segs = np.array([[0, 2, 5], [3, 4, 30], [4, 5, 0]], dtype=np.uint32)
    mask, lst = orc.select(imp, segs)
    per = 24
    assert mask[0:2].sum() == 5 and mask[2].sum() == 0 and mask[3].sum() == 24 and mask[4].sum() == 0
    sel = imp[0:2].ravel()[mask[0:2].ravel() == 1]
    rest = imp[0:2].ravel()[mask[0:2].ravel() == 0]
    assert sel.min() >= rest.max()
    assert np.array_equal(lst, np.flatnonzero(mask.ravel()))
    with pytest.raises(ValueError):
        orc.select(imp, np.array([[0, 3, 1], [2, 4, 1]], dtype=np.uint32))   # overlap
    with pytest.raises(ValueError):
        orc.select(imp, np.array([[0, 6, 1]], dtype=np.uint32))              # out of range
    assert per * 5 == imp.size


def test_threshold_closed_form(orc):
    rng = np.random.default_rng(4)
    imp = rng.random((3, 5, 7)).astype(np.float32)
    imp[1, 2, 3] = np.nan
    imp[0, 0, 0] = 0.5
    segs = np.array([[0, 2, 0], [2, 3, 0]], dtype=np.uint32)
    thr = np.array([0.5, 0.9], dtype=np.float32)
    mask, lst = orc.select(imp, segs, "threshold", thr)
    with np.errstate(invalid="ignore"):
        want = np.concatenate([(imp[0:2] >= 0.5).ravel(), (imp[2:3] >= np.float32(0.9)).ravel()])
    assert np.array_equal(mask.ravel().astype(bool), want)
    assert mask[0, 0, 0] == 1 and mask[1, 2, 3] == 0
    assert np.array_equal(lst, np.flatnonzero(want))


def test_budget_by_hand(orc):
    # largest N with 256 N <= H W B (Sec. 3.3.1)
    assert orc.budget(128, 128, 1) == 64
    assert orc.budget(64, 64, 3) == 48
    assert orc.budget(96, 96, 1) == 36
    assert orc.budget(100, 100, 1) == 39        # 10000/256 = 39.06
    for (h, w, b) in [(128, 128, 7), (90, 70, 3)]:
        n = orc.budget(h, w, b)
        assert 256 * n <= h * w * b < 256 * (n + 1)
