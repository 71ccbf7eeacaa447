"""Pins of the temporal-reuse oracle (Sec. 3.2.2): hand cases, a library labelling routine as
second opinion, closed-form frame choices, exact rationals, and a textbook apportionment."""
from fractions import Fraction

import numpy as np
import pytest
from scipy import ndimage

import workloads as wl
from oracle import temporal as T

ONE = 1 << 32


def frame_with(rects, H=24, W=32, val=50):
    r = np.zeros((H, W), dtype=np.int16)
    for (y, x, h, w) in rects:
        r[y:y + h, x:x + w] = val
    return r


def phi1(img, tau=10, min_area=1):
    p, nb = T.phi(img[None], tau, min_area)
    return int(p[0]), int(nb[0])


def test_phi_hand_cases():
    assert phi1(frame_with([])) == (0, 0)
    assert phi1(frame_with([(3, 4, 2, 5)])) == (ONE // 10, 1)                       # one 2x5 blob
    assert phi1(frame_with([(0, 0, 1, 1)])) == (ONE, 1)                             # a single corner pixel
    assert phi1(frame_with([(1, 1, 3, 3), (10, 10, 2, 2)])) == (ONE // 9 + ONE // 4, 2)
    # diagonal contact joins two blobs (8-neighbourhood); one pixel further apart they stay two
    assert phi1(frame_with([(2, 2, 2, 2), (4, 4, 2, 2)])) == (ONE // 8, 1)
    assert phi1(frame_with([(2, 2, 2, 2), (5, 5, 2, 2)])) == (2 * (ONE // 4), 2)
    # anti-diagonal contact too
    assert phi1(frame_with([(4, 2, 2, 2), (2, 4, 2, 2)])) == (ONE // 8, 1)
    # the whole frame is one blob
    assert phi1(frame_with([(0, 0, 24, 32)])) == (ONE // (24 * 32), 1)


def test_phi_threshold_is_strict_and_uses_the_magnitude():
    img = np.zeros((8, 8), dtype=np.int16)
    img[1, 1] = 10; img[3, 3] = 11; img[5, 5] = -11; img[7, 7] = -10
    assert phi1(img, tau=10) == (2 * ONE, 2)
    assert phi1(img, tau=9) == (4 * ONE, 4)
    assert phi1(img, tau=11) == (0, 0)


def test_phi_min_area_drops_small_blobs():
    img = frame_with([(1, 1, 1, 1), (5, 5, 2, 2), (10, 10, 3, 3)])
    assert phi1(img, min_area=1) == (ONE + ONE // 4 + ONE // 9, 3)
    assert phi1(img, min_area=2) == (ONE // 4 + ONE // 9, 2)
    assert phi1(img, min_area=4) == (ONE // 4 + ONE // 9, 2)
    assert phi1(img, min_area=5) == (ONE // 9, 1)
    assert phi1(img, min_area=10) == (0, 0)


def test_phi_winding_blob_is_one_blob():
    # a one-pixel-wide serpentine: a labelling that only looks up/left once would split it
    H, W = 17, 21
    img = np.zeros((H, W), dtype=np.int16)
    for y in range(0, H, 2):
        img[y, :] = 40
        if y + 1 < H:
            img[y + 1, W - 1 if (y // 2) % 2 == 0 else 0] = 40
    area = int((img != 0).sum())
    assert phi1(img) == (ONE // area, 1)
    # a ring and the dot inside it are two blobs
    ring = frame_with([(2, 2, 9, 9)]); ring[4:9, 4:9] = 0; ring[6, 6] = 50
    assert phi1(ring) == (ONE // (81 - 25) + ONE, 2)


@pytest.mark.parametrize("density", [0.02, 0.2, 0.45, 0.6, 0.9])
def test_phi_against_library_labelling(density):
    rng = np.random.default_rng(int(density * 100))
    res = (rng.random((3, 37, 53)) < density).astype(np.int16) * rng.integers(20, 200, (3, 37, 53)).astype(np.int16)
    res *= rng.choice(np.array([-1, 1], dtype=np.int16), size=res.shape)
    for min_area in (1, 3):
        got, nb = T.phi(res, 10, min_area)
        for f in range(3):
            lab, n = ndimage.label(np.abs(res[f]) > 10, structure=np.ones((3, 3)))
            areas = np.bincount(lab.ravel())[1:]
            areas = areas[areas >= min_area]
            assert int(got[f]) == sum(ONE // int(a) for a in areas)
            assert int(nb[f]) == len(areas)


def test_phi_frames_are_independent_and_on_the_synthetic_residuals():
    res = wl.make_residuals(96, 64, 2, 3, seed=3)
    whole, _ = T.phi(res, 12, 2)
    for f in range(len(res)):
        assert int(T.phi(res[f:f + 1], 12, 2)[0][0]) == int(whole[f])
    # second opinion on the workload's own value distribution
    for f in range(len(res)):
        lab, n = ndimage.label(np.abs(res[f].astype(np.int32)) > 12, structure=np.ones((3, 3)))
        areas = np.bincount(lab.ravel())[1:]
        assert int(whole[f]) == sum(ONE // int(a) for a in areas if a >= 2)


def test_inverse_area_responds_to_small_objects_and_area_to_large_blocks():
    """The property the paper's appendix on operators illustrates: a large changed block moves
    the area feature a lot and the inverse-area feature hardly; small objects do the opposite."""
    H, W = 90, 160
    big = frame_with([(10, 10, 60, 120)], H, W)
    small = frame_with([(5, 5, 4, 4), (30, 80, 5, 3), (60, 20, 3, 6), (70, 140, 4, 5), (40, 40, 2, 7)], H, W)
    area = lambda img: float((img != 0).sum()) / (H * W)
    p_big, p_small = phi1(big)[0] / ONE, phi1(small)[0] / ONE
    assert area(big) > 10 * area(small)
    assert p_small > 100 * p_big


# ---- frame choice -------------------------------------------------------------------------

def test_uniform_change_picks_evenly_spaced_frames():
    ph = [7 * i for i in range(9)]                     # 8 equal steps: positions f/8
    picks, reuse = T.frame_select(ph, 4)
    assert picks == [1, 3, 5, 7]                       # positions 1/8, 3/8, 5/8, 7/8 = the midpoints
    assert reuse == [1, 1, 3, 3, 5, 5, 7, 7, 7]
    # decreasing Phi changes nothing: the magnitude of the change counts
    assert T.frame_select(ph[::-1], 4) == (picks, reuse)
    # neither does an offset or a scale of Phi
    assert T.frame_select([1000 + 3 * v for v in ph], 4) == (picks, reuse)


def test_a_single_jump_predicts_the_first_frame_and_the_frame_after_the_jump():
    ph = [5, 5, 5, 5, 5, 90, 90, 90, 90]
    picks, reuse = T.frame_select(ph, 2)
    assert picks == [0, 5]
    assert reuse == [0, 0, 0, 0, 0, 5, 5, 5, 5]
    # more intervals than distinct positions: the empty ones select nothing
    assert T.frame_select(ph, 7)[0] == [0, 5]


def test_no_change_at_all_predicts_only_the_first_frame():
    assert T.frame_select([3] * 6, 4) == ([0], [0] * 6)
    assert T.frame_select([3], 1) == ([0], [0])


def test_one_interval_takes_the_frame_nearest_the_middle_of_the_change():
    ph = [0, 1, 2, 4, 8, 16]                           # positions 0, 1/16, 2/16, 4/16, 8/16, 1
    assert T.frame_select(ph, 1) == ([4], [4] * 6)
    ph = [0, 6, 10, 16]                                # 6/16 and 10/16: equally near, earlier wins
    assert T.frame_select(ph, 1) == ([1], [1] * 4)


def test_as_many_intervals_as_steps_with_uniform_change():
    ph = list(range(9))
    picks, reuse = T.frame_select(ph, 8)
    assert picks == list(range(8))                     # frames 7 and 8 share the last interval, 7 is as near
    assert reuse == [0, 1, 2, 3, 4, 5, 6, 7, 7]


@pytest.mark.parametrize("seed", range(20))
def test_frame_choice_against_exact_rationals(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 40))
    N = int(rng.integers(1, 12))
    ph = [int(v) for v in rng.integers(0, 1 << 40, n)]
    if seed % 4 == 0:                                  # plateaus: many equal positions
        ph = [ph[i - i % 3] for i in range(n)]
    picks, reuse = T.frame_select(ph, N)
    S = [abs(ph[i + 1] - ph[i]) for i in range(n - 1)]
    tot = sum(S)
    P = [Fraction(sum(S[:f]), tot) if tot else Fraction(0) for f in range(n)]
    cell = [min(N - 1, int(p * N)) for p in P]         # int() floors a non-negative Fraction
    want = {}
    for j in set(cell):
        members = [f for f in range(n) if cell[f] == j]
        want[j] = min(members, key=lambda f: (abs(P[f] - Fraction(2 * j + 1, 2 * N)), f))
    assert picks == sorted(want.values())
    assert reuse == [want[cell[f]] for f in range(n)]
    # invariants: at most N picks, every pick reuses itself, intervals are runs of frames
    assert len(picks) <= N and all(reuse[p] == p for p in picks)
    assert cell == sorted(cell)


# ---- budget over streams --------------------------------------------------------------------

def test_allocate_hand_cases():
    assert T.allocate([50, 30, 20], 13) == [6, 4, 3]          # 1 each + 10 shared 5/3/2
    assert T.allocate([1, 1, 1], 5) == [2, 2, 1]              # equal remainders: lower streams first
    assert T.allocate([0, 0, 0], 8) == [3, 3, 2]              # nothing changed anywhere: equal shares
    assert T.allocate([0, 9, 0], 6) == [1, 4, 1]              # a still stream keeps its one frame
    assert T.allocate([4, 4], 2) == [1, 1]
    with pytest.raises(ValueError):
        T.allocate([1, 2, 3], 2)


def test_allocate_is_largest_remainder_apportionment():
    # the classic example of this method (three states with populations 6, 6, 2): 10 seats go
    # 4, 4, 2 and 11 seats go 5, 5, 1
    assert T.allocate([6, 6, 2], 3 + 10) == [5, 5, 3]
    assert T.allocate([6, 6, 2], 3 + 11) == [6, 6, 2]


@pytest.mark.parametrize("seed", range(10))
def test_allocate_properties(seed):
    rng = np.random.default_rng(100 + seed)
    ns = int(rng.integers(1, 12))
    tot = [int(v) for v in rng.integers(0, 1 << 50, ns)]
    n_total = ns + int(rng.integers(0, 60))
    a = T.allocate(tot, n_total)
    assert sum(a) == n_total and min(a) >= 1
    whole = sum(tot)
    for s in range(ns):                                       # within one of the exact share
        share = Fraction((n_total - ns) * tot[s], whole) if whole else Fraction(n_total - ns, ns)
        assert abs(a[s] - 1 - share) < 1
    for s in range(ns):
        for t in range(ns):
            if tot[s] > tot[t]:
                assert a[s] >= a[t]


def test_temporal_plan_and_spread_on_streams():
    res = wl.make_residuals(96, 64, 3, 6, seed=1)
    ph, _ = T.phi(res, 12, 2)
    off = [0, 6, 12, 18]
    alloc, sel, reuse = T.temporal_plan(ph, off, 8)
    assert sum(alloc) == 8
    for s in range(3):
        b, e = off[s], off[s + 1]
        assert 1 <= sel[b:e].sum() <= alloc[s]
        assert all(b <= r < e for r in reuse[b:e])            # never reuse across streams
    assert all(sel[r] == 1 for r in reuse) and all(reuse[f] == f for f in np.flatnonzero(sel))
    imp = np.arange(18 * 4 * 6, dtype=np.float32).reshape(18, 4, 6)
    out = T.spread(imp, reuse)
    for f in range(18):
        assert np.array_equal(out[f], imp[reuse[f]])
