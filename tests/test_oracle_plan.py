"""Pins for the oracle's packing plan (Alg. 1, Appx. A) that do not call the oracle's own
arithmetic: library labelling, exact rationals, an O(n^2) validity check, an independent
re-simulation of the first-fit rules, and a hand-traced example."""
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest
from scipy import ndimage

import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden")
ST8 = np.ones((3, 3), dtype=int)
ST4 = np.array([[0, 1, 0], [1, 1, 1], [0, 1, 0]])


def owned_sets(plan, mask):
    """box index -> set of owned flat ids, from the placement rows."""
    own = {}
    for g, box, *_ in plan.places.tolist():
        own.setdefault(box, set()).add(g)
    assert sorted(g for s in own.values() for g in s) == np.flatnonzero(mask.ravel()).tolist()
    return own


def check_valid(plan, mask, imp, halo, S, T, conn, sort_policy="density", rotate=False):
    """Everything that must hold for any correct run, checked by brute force."""
    F, mbh, mbw = mask.shape
    per = mbh * mbw
    own = owned_sets(plan, mask)
    assert set(own) == set(range(len(plan.boxes)))                      # no empty boxes
    lab = [ndimage.label(mask[f], structure=ST8 if conn == 8 else ST4)[0] for f in range(F)]
    rects = []
    for i, (f, x0, y0, w, h, rot, b, bx, by, bid) in enumerate(plan.boxes.tolist()):
        gs = sorted(own[i])
        assert bid == gs[0] and rot in ((0, 1) if rotate else (0,))
        xs = [g % mbw for g in gs]; ys = [(g % per) // mbw for g in gs]
        assert all(g // per == f for g in gs)
        assert (min(xs), min(ys), max(xs) - min(xs) + 1, max(ys) - min(ys) + 1) == (x0, y0, w, h)  # tight
        assert w <= T and h <= T
        assert len({lab[f][y, x] for x, y in zip(xs, ys)}) == 1             # one region per box
        bw, bh = 16 * w + 2 * halo, 16 * h + 2 * halo
        if rot:
            bw, bh = bh, bw                                                   # occupied size
        if b != 0xFFFF:
            assert 0 <= b < plan.n_bins and bx >= 0 and by >= 0 and bx + bw <= S and by + bh <= S
            rects.append((b, bx, by, bw, bh))
    for (b1, x1, y1, w1, h1), (b2, x2, y2, w2, h2) in itertools.combinations(rects, 2):
        if b1 == b2:
            assert x1 + w1 <= x2 or x2 + w2 <= x1 or y1 + h1 <= y2 or y2 + h2 <= y1, "boxes overlap"
    # density order, in exact rational arithmetic on the fp32 canonical sum
    keys = []
    for i, row in enumerate(plan.boxes.tolist()):
        s = np.float32(0)
        for g in sorted(own[i]):
            s = np.float32(s + imp.ravel()[g])
        if sort_policy == "area":
            keys.append((-row[3] * row[4], row[9]))
        else:
            keys.append((-Fraction(float(s)) / (row[3] * row[4]), row[9]))
    assert keys == sorted(keys)
    # placement rows
    for j, (g, box, b, px, py) in enumerate(plan.places.tolist()):
        f, x0, y0, w, h, rot, bb, bx, by, bid = plan.boxes[box].tolist()
        assert b == bb and plan.place_rot[j] == rot
        dx, dy = halo + 16 * (g % mbw - x0), halo + 16 * ((g % per) // mbw - y0)
        assert (px, py) == ((bx + dy, by + dx) if rot else (bx + dx, by + dy))
    # MBs of one region that fall in the same T-cell of the region's bbox share a box
    for f in range(F):
        for r in range(1, lab[f].max() + 1):
            ys, xs = np.nonzero(lab[f] == r)
            cell = {}
            for y, x in zip(ys, xs):
                key = ((x - xs.min()) // T, (y - ys.min()) // T)
                g = f * per + y * mbw + x
                bx_ = [i for i, s in own.items() if g in s][0]
                assert cell.setdefault(key, bx_) == bx_
            assert len(set(cell.values())) == len(cell)


def simulate_first_fit(sizes, halo, S, max_bins=1 << 15, rotate=False):
    """Independent re-simulation of the placement rules from their prose statement."""
    m = 16 + 2 * halo
    free, out, nb = [], [], 0
    for (bw, bh) in sizes:
        def fits(r):
            return (r[3] >= bw and r[4] >= bh) or (rotate and r[3] >= bh and r[4] >= bw)
        idx = next((i for i, r in enumerate(free) if fits(r)), None)
        if idx is None:
            if nb >= max_bins:
                break
            free.append((nb, 0, 0, S, S)); idx = len(free) - 1; nb += 1
        b, x, y, w, h = free[idx]
        turned = not (w >= bw and h >= bh)
        if turned:
            bw, bh = bh, bw
        out.append((b, x, y, int(turned)) if rotate else (b, x, y))
        if (w - bw) * h >= w * (h - bh):
            right, bottom = (b, x + bw, y, w - bw, h), (b, x, y + bh, bw, h - bh)
        else:
            right, bottom = (b, x + bw, y, w - bw, bh), (b, x, y + bh, w, h - bh)
        new = [r for r in (right, bottom) if r[3] >= m and r[4] >= m]
        new.sort(key=lambda r: r[3] * r[4])           # stable: right before bottom on ties
        free[idx:idx + 1] = new
    return out, nb, free


def check_against_simulation(plan, halo, S, max_bins=1 << 15, rotate=False):
    sizes = [(16 * r[3] + 2 * halo, 16 * r[4] + 2 * halo) for r in plan.boxes.tolist()]
    out, nb, free = simulate_first_fit(sizes, halo, S, max_bins, rotate)
    if rotate:
        got = [(r[6], r[7], r[8], r[5]) for r in plan.boxes.tolist() if r[6] != 0xFFFF]
        sizes = [(h, w) if o[3] else (w, h) for (w, h), o in zip(sizes, out)]     # occupied sizes
        out3 = [o[:3] for o in out]
    else:
        got = [(r[6], r[7], r[8]) for r in plan.boxes.tolist() if r[6] != 0xFFFF]
        out3 = out
    assert got == out and nb == plan.n_bins
    out = out3
    # area conservation: free + placed + dropped slivers = n_bins * S^2  =>  free + placed <= total
    placed = sum(w * h for (w, h), _ in zip(sizes, out))
    assert placed + sum(r[3] * r[4] for r in free) <= nb * S * S
    # free rects are disjoint from boxes of the same bin
    for (b, x, y, w, h) in free:
        for (bw, bh), (bb, bx, by) in zip(sizes, out):
            if bb == b:
                assert x + w <= bx or bx + bw <= x or y + h <= by or by + bh <= y


def test_labelling_all_3x3_masks_vs_library(orc):
    for conn in (4, 8):
        for bits in range(512):
            mask = np.array([(bits >> i) & 1 for i in range(9)], dtype=np.uint8).reshape(1, 3, 3)
            imp = np.ones((1, 3, 3), dtype=np.float32)
            pl = orc.plan(mask, imp, halo=2, bin_size=128, conn=conn, T=6)
            lab, n = ndimage.label(mask[0], structure=ST8 if conn == 8 else ST4)
            assert len(pl.boxes) == n
            want = sorted((sl[1].start, sl[0].start, sl[1].stop - sl[1].start, sl[0].stop - sl[0].start)
                          for sl in ndimage.find_objects(lab))
            assert sorted(tuple(r[1:5]) for r in pl.boxes.tolist()) == want


@pytest.mark.parametrize("seed", range(12))
def test_random_masks_valid_and_first_fit(orc, seed):
    rng = np.random.default_rng(seed)
    F, mbh, mbw = 3, 6 + seed % 3, 7
    mask = (rng.random((F, mbh, mbw)) < [0.2, 0.45, 0.7][seed % 3]).astype(np.uint8)
    imp = rng.random((F, mbh, mbw)).astype(np.float32)
    if seed % 4 == 0:
        imp = np.floor(imp * 3).astype(np.float32)      # heavy ties
    for conn, T, halo, S in [(8, 3, 4, 64), (4, 2, 3, 64), (8, 5, 6, 96), (8, 1, 10, 128)]:
        pl = orc.plan(mask, imp, halo, S, conn, T)
        assert not pl.overflow
        check_valid(pl, mask, imp, halo, S, T, conn)
        check_against_simulation(pl, halo, S)


def test_hand_cases(orc):
    imp = np.ones((1, 5, 5), dtype=np.float32)
    diag = np.zeros((1, 5, 5), dtype=np.uint8); diag[0, 1, 1] = diag[0, 2, 2] = 1
    assert len(orc.plan(diag, imp, 4, 64, 8, 3).boxes) == 1
    assert len(orc.plan(diag, imp, 4, 64, 4, 3).boxes) == 2
    ring = np.zeros((1, 5, 5), dtype=np.uint8); ring[0] = 1; ring[0, 1:4, 1:4] = 0; ring[0, 2, 2] = 1
    pl = orc.plan(ring, imp, 4, 128, 8, 6)
    rows = sorted(tuple(r[1:5]) for r in pl.boxes.tolist())
    assert rows == [(0, 0, 5, 5), (2, 2, 1, 1)]                       # nested bounding boxes
    dens = {tuple(r[1:5]): i for i, r in enumerate(pl.boxes.tolist())}
    assert dens[(2, 2, 1, 1)] < dens[(0, 0, 5, 5)]                    # density 1 before 16/25
    # the ring's box covers the dot but does not own it
    own = owned_sets(pl, ring)
    assert 12 not in own[dens[(0, 0, 5, 5)]] and own[dens[(2, 2, 1, 1)]] == {12}
    # L-shape cut with T=2: 3x3 L -> cells tightened, empty cell dropped
    L = np.zeros((1, 5, 5), dtype=np.uint8); L[0, 0:3, 0] = 1; L[0, 2, 0:3] = 1
    pl = orc.plan(L, imp, 4, 64, 8, 2)
    assert sorted(tuple(r[1:5]) for r in pl.boxes.tolist()) == [(0, 0, 1, 2), (0, 2, 2, 1), (2, 2, 1, 1)]
    check_valid(pl, L, imp, 4, 64, 2, 8)


def test_empty_single_and_overflow(orc):
    imp = np.ones((2, 4, 4), dtype=np.float32)
    none = np.zeros((2, 4, 4), dtype=np.uint8)
    pl = orc.plan(none, imp, 4, 64)
    assert len(pl.boxes) == 0 and pl.n_bins == 0 and len(pl.places) == 0 and not pl.overflow
    one = none.copy(); one[1, 3, 2] = 1
    pl = orc.plan(one, imp, 4, 64)
    assert pl.boxes.tolist() == [[1, 2, 3, 1, 1, 0, 0, 0, 0, 30]] and pl.n_bins == 1
    assert pl.places.tolist() == [[30, 0, 0, 4, 4]]
    # 16 isolated MBs, 4 per 64-bin -> 4 bins; allow only 2
    iso = np.zeros((1, 8, 8), dtype=np.uint8); iso[0, ::2, ::2] = 1
    imp8 = np.arange(64, dtype=np.float32).reshape(1, 8, 8)
    pl = orc.plan(iso, imp8, 4, 64, max_bins=2)
    assert pl.overflow and pl.n_bins == 2
    assert [r[6] for r in pl.boxes.tolist()] == [0] * 4 + [1] * 4 + [0xFFFF] * 8
    check_against_simulation(pl, 4, 64, max_bins=2)
    with pytest.raises(ValueError):
        orc.plan(iso, imp8, 30, 64)           # 16 + 2*30 > 64


def test_golden_hand_trace(orc):
    rows = [ln.split("#")[0].split() for ln in open(os.path.join(GOLD, "firstfit_five_boxes.txt"))
            if ln.strip() and not ln.startswith("#")]
    want = [(int(r[1]), int(r[2]), int(r[3])) for r in rows]
    mask = np.zeros((1, 6, 6), dtype=np.uint8)
    for (y, x) in [(0, 0), (0, 2), (0, 4), (2, 0), (2, 2)]:
        mask[0, y, x] = 1
    imp = np.full((1, 6, 6), 0.5, dtype=np.float32)
    pl = orc.plan(mask, imp, halo=4, bin_size=64)
    assert [(r[6], r[7], r[8]) for r in pl.boxes.tolist()] == want
    assert [r[9] for r in pl.boxes.tolist()] == [0, 2, 4, 12, 14]
    # the free lists written in the fixture, via the independent simulation
    out, nb, free = simulate_first_fit([(24, 24)] * 5, 4, 64)
    assert out == want and nb == 2 and free == [(1, 0, 24, 24, 40), (1, 24, 0, 40, 64)]


@pytest.mark.parametrize("ci", [1, 2, 3, 5])
def test_benchmark_configs_plan_valid(orc, ci):
    cfg = wl.config(ci)
    imp = wl.make_importance(cfg)
    mask, lst = orc.select(imp, wl.make_segments(cfg))
    T = (cfg.bin_size - 2 * cfg.halo) // 16
    pl = orc.plan(mask, imp, cfg.halo, cfg.bin_size)
    assert not pl.overflow and len(pl.places) == len(lst)
    check_against_simulation(pl, cfg.halo, cfg.bin_size)
    if ci <= 2:
        check_valid(pl, mask, imp, cfg.halo, cfg.bin_size, T, 8)
    occ = 256 * len(lst) / (pl.n_bins * cfg.bin_size ** 2)
    assert 0.1 < occ <= 1.0


@pytest.mark.parametrize("seed", range(8))
def test_policy_options_valid_and_first_fit(orc, seed):
    """Large-item-first order and RotatePacking (Alg. 1): same brute-force validity checks and the
    independent re-simulation, with the option switched on on both sides."""
    rng = np.random.default_rng(100 + seed)
    F, mbh, mbw = 4, 7, 9
    mask = (rng.random((F, mbh, mbw)) < [0.15, 0.3, 0.5, 0.7][seed % 4]).astype(np.uint8)
    imp = rng.random((F, mbh, mbw)).astype(np.float32)
    n_rot = 0
    for conn, T, halo, S in [(8, 3, 4, 64), (4, 4, 3, 80), (8, 5, 6, 96), (8, 6, 10, 128)]:
        for policy, rotate in (("area", False), ("density", True), ("area", True)):
            pl = orc.plan(mask, imp, halo, S, conn, T, sort_policy=policy, rotate=rotate)
            assert not pl.overflow
            check_valid(pl, mask, imp, halo, S, T, conn, policy, rotate)
            check_against_simulation(pl, halo, S, rotate=rotate)
            n_rot += int(pl.boxes[:, 5].sum())
    assert n_rot > 0                                    # the turned branch is exercised


def test_rotate_hand_traced(orc):
    """tests/golden/rotate_three_boxes.txt: a 40x24 box, a 40x40 box and another 40x24 box in a 64x64
    bin with halo 4; the third only fits the 24x40 remainder when turned (traced by hand)."""
    mask = np.zeros((3, 3, 3), dtype=np.uint8); imp = np.zeros((3, 3, 3), dtype=np.float32)
    mask[0, 0, 0:2] = 1; imp[0, 0, 0:2] = 0.9
    mask[1, 0:2, 0:2] = 1; imp[1, 0:2, 0:2] = 0.5
    mask[2, 0, 0:2] = 1; imp[2, 0, 0:2] = 0.2
    rows = [tuple(int(v) for v in ln.split()) for ln in open(os.path.join(GOLD, "rotate_three_boxes.txt"))
            if ln.strip() and not ln.startswith("#")]
    want_rot = [r[1:] for r in rows if r[0] == 1]       # (bin, bx, by, rot) per box, rotation on
    want_off = [r[1:] for r in rows if r[0] == 0]
    want_pl = [r[1:] for r in rows if r[0] == 2]        # (mb_id, px, py) of the turned box's MBs
    pl = orc.plan(mask, imp, 4, 64, 8, 3, rotate=True)
    assert [(r[6], r[7], r[8], r[5]) for r in pl.boxes.tolist()] == want_rot and pl.n_bins == 1
    got = {g: (px, py) for g, box, b, px, py in pl.places.tolist()}
    assert all(got[g] == (px, py) for g, px, py in want_pl)
    pl0 = orc.plan(mask, imp, 4, 64, 8, 3, rotate=False)
    assert [(r[6], r[7], r[8], r[5]) for r in pl0.boxes.tolist()] == want_off and pl0.n_bins == 2


def test_area_policy_order_differs_from_density(orc):
    """A large sparse box and a small dense one: density-first packs the small one first,
    large-item-first the large one (the comparison of Sec. 3.3.2)."""
    mask = np.zeros((1, 4, 8), dtype=np.uint8); imp = np.zeros((1, 4, 8), dtype=np.float32)
    mask[0, 0, 0] = mask[0, 1, 1] = mask[0, 2, 2] = 1; imp[0, 0, 0] = imp[0, 1, 1] = imp[0, 2, 2] = 0.3   # 3x3 bbox
    mask[0, 0, 6] = 1; imp[0, 0, 6] = 0.9
    d = orc.plan(mask, imp, 4, 128, 8, 6)
    a = orc.plan(mask, imp, 4, 128, 8, 6, sort_policy="area")
    assert [r[3] * r[4] for r in d.boxes.tolist()] == [1, 9]
    assert [r[3] * r[4] for r in a.boxes.tolist()] == [9, 1]
