"""Planner-lite: choose the enhancer's tensor sizes from a measured cost curve (Sec. 3.4).

The paper's execution planner assigns every component its input tensor size: for a component
with cost curve c(b) (time of one launch on b inputs) it takes, within the time budget r', the
size that maximises b / c(b) (the inner term of the Sec. 3.4 recurrence).  For the region-aware
enhancer the tensor is the bin batch, so the knobs are the bin side S (Sec. 3.3.1 fixes the
macroblock budget as S*S*B / 256), the partition's preset size (the largest box side in
macroblocks) and the number of bins per launch.  This module is host logic only and runs outside
the hot path:

  * `choose(curve, candidates, ...)`: given the measured curve and, for every candidate geometry,
    how many bins the workload's batch needs, return the geometry and launch size with the highest
    enhanced-macroblock rate;
  * `measure_curve(...)` / `measure_candidates(...)`: produce those inputs on the GPU with the
    library itself (rh_enhance timed with the library's event brackets, rh_pack's bin count);
  * `python -m paper_2407_16990_amd.planner --measure OUT.json` writes the table that is kept in
    the tree as planner_curve_mi355x.json.
"""
from __future__ import annotations

import json
import math
import os
from dataclasses import dataclass
from typing import Dict, Iterable, List, Optional, Sequence, Tuple

CURVE_FILE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "planner_curve_mi355x.json")


def cost(points: Sequence[Tuple[int, float]], b: int) -> float:
    """c(b): time (ms) of one launch on b bins, from measured (b, ms) points: linear between the
    points, proportional below the first and along the last segment's slope above the last."""
    pts = sorted((int(p[0]), float(p[1])) for p in points)
    if not pts or b < 0:
        raise ValueError("cost: empty curve or negative batch")
    if b == 0:
        return 0.0
    if b <= pts[0][0]:
        # a launch never costs less than its fixed part: hold the first point's cost per launch
        # for smaller batches (conservative: small launches do not get cheaper than measured)
        return pts[0][1]
    for (b0, c0), (b1, c1) in zip(pts, pts[1:]):
        if b <= b1:
            return c0 + (c1 - c0) * (b - b0) / (b1 - b0)
    if len(pts) == 1:
        return pts[0][1] * b / pts[0][0]
    (b0, c0), (b1, c1) = pts[-2], pts[-1]
    return c1 + (c1 - c0) / (b1 - b0) * (b - b1)


def best_launch_size(points: Sequence[Tuple[int, float]], b_max: int, budget_ms: Optional[float] = None) -> int:
    """argmax over 1 <= b <= b_max with c(b) <= budget of b / c(b); ties go to the smaller b
    (lower latency).  0 when no size fits the budget."""
    best, best_rate = 0, -1.0
    for b in range(1, max(b_max, 0) + 1):
        c = cost(points, b)
        if budget_ms is not None and c > budget_ms:
            continue
        rate = b / c
        if rate > best_rate * (1.0 + 1e-12):
            best, best_rate = b, rate
    return best


@dataclass(frozen=True)
class Candidate:
    """One geometry and what the workload's batch needs under it (from the packer itself)."""
    bin_size: int
    max_box_mbs: int      # 0 = the largest box that fits a bin
    n_bins: int           # bins the batch packs into
    n_selected: int       # macroblocks enhanced


@dataclass(frozen=True)
class Choice:
    bin_size: int
    max_box_mbs: int
    bins_per_launch: int
    launches: int
    ms_per_batch: float
    macroblocks_per_s: float


def batch_time(points: Sequence[Tuple[int, float]], n_bins: int, per_launch: int) -> Tuple[float, int]:
    """Time to enhance n_bins bins in launches of at most per_launch bins -> (ms, launches)."""
    if n_bins == 0:
        return 0.0, 0
    full, rest = divmod(n_bins, per_launch)
    ms = full * cost(points, per_launch) + (cost(points, rest) if rest else 0.0)
    return ms, full + (1 if rest else 0)


def choose(curve: Dict[int, Sequence[Tuple[int, float]]], candidates: Iterable[Candidate],
           budget_ms: Optional[float] = None, other_ms: float = 0.0) -> Choice:
    """The candidate with the highest enhanced-macroblock rate.

    curve[S]: measured (bins, ms) points of rh_enhance on S x S bins; budget_ms: latency budget of
    one launch (None = unbounded); other_ms: time of the batch's other steps (selection, packing,
    paste), taken as independent of the geometry.  For every candidate the launch size is the one
    that maximises b / c(b) within the budget (never more than the batch needs); a whole batch in
    one launch is kept whenever splitting it does not raise the rate.  Ties: smaller bins first,
    then the larger preset size."""
    best: Optional[Choice] = None
    for cand in sorted(candidates, key=lambda c: (c.bin_size, -c.max_box_mbs if c.max_box_mbs else -10 ** 9)):
        if cand.bin_size not in curve:
            raise KeyError(f"no measured curve for bin size {cand.bin_size}")
        pts = curve[cand.bin_size]
        if cand.n_bins == 0:
            continue
        per = best_launch_size(pts, cand.n_bins, budget_ms)
        if per == 0:
            continue                                       # not even one bin fits the budget
        ms, launches = batch_time(pts, cand.n_bins, per)
        one = cost(pts, cand.n_bins)                       # the whole batch at once, if the budget allows
        if (budget_ms is None or one <= budget_ms) and one <= ms:
            ms, launches, per = one, 1, cand.n_bins
        total = ms + other_ms
        rate = cand.n_selected / (total * 1e-3) if total > 0 else 0.0
        c = Choice(cand.bin_size, cand.max_box_mbs, per, launches, total, rate)
        if best is None or c.macroblocks_per_s > best.macroblocks_per_s * (1.0 + 1e-9):
            best = c
    if best is None:
        raise ValueError("choose: no candidate fits the latency budget")
    return best


# ---------------------------------------------------------------------------------------------
# measuring the inputs on the GPU (needs the library and a device; not used by choose())

def measure_curve(net, weights, precision: str, bin_sizes: Sequence[int], batches: Sequence[int], halo: int,
                  reps: int = 5) -> Dict[int, List[Tuple[int, float]]]:
    """c(b) of rh_enhance for every bin size: median over reps of the event-bracketed kernel time."""
    import torch
    from .binding import RH
    out: Dict[int, List[Tuple[int, float]]] = {}
    for S in bin_sizes:
        rh = RH(frame_w=max(64, S), frame_h=max(64, S), max_frames=1, halo=halo, bin_size=S, max_bins=max(batches),
                net=net, weights=weights, precision=precision)
        pts = []
        for b in batches:
            bins = torch.randint(0, 256, (b, S, S, 3), dtype=torch.uint8, device="cuda")
            res = torch.empty((b, S * net.scale, S * net.scale, 3), dtype=torch.float32, device="cuda")
            rh.enhance(bins, out=res)                      # warm-up, workspace allocation
            times = []
            for _ in range(reps):
                rh.profile_enable(True); rh.profile_read()
                rh.enhance(bins, out=res)
                p = rh.profile_read(); rh.profile_enable(False)
                times.append(p["head"][0] + p["conv"][0] + p["conv_last"][0])
            pts.append((int(b), float(sorted(times)[len(times) // 2])))
            del bins, res
        out[int(S)] = pts
        rh.close()
    return out


def measure_candidates(frames, importance, segments, net, weights, precision: str, halo: int,
                       geometries: Sequence[Tuple[int, int]], max_bins: int = 4096) -> List[Candidate]:
    """Runs the selection and the packer on the workload's batch for every (bin_size, max_box_mbs)."""
    from .binding import RH
    cands = []
    F, H, W, _ = frames.shape
    for S, T in geometries:
        rh = RH(frame_w=W, frame_h=H, max_frames=F, halo=halo, bin_size=S, max_bins=max_bins, net=net, weights=weights,
                precision=precision, max_box_mbs=T)
        mask, lst, n_sel = rh.select_regions(importance, segments)
        po = rh.pack(frames, importance, mask, lst, n_sel)
        n_boxes, n_bins, _, k = rh.read_counts(po.counts)
        cands.append(Candidate(int(S), int(T), int(n_bins), int(k)))
        rh.close()
    return cands


def load_curve(path: str = CURVE_FILE) -> Dict[int, List[Tuple[int, float]]]:
    with open(path) as f:
        d = json.load(f)
    return {int(S): [(int(b), float(ms)) for b, ms in pts] for S, pts in d["curve"].items()}


def main(argv=None) -> int:
    import argparse
    ap = argparse.ArgumentParser(description="measure the enhancer's cost curve c(b) on this GPU")
    ap.add_argument("--measure", metavar="OUT.json", required=True)
    ap.add_argument("--config", type=int, default=3)
    ap.add_argument("--bin-sizes", type=int, nargs="+", default=[96, 128, 160, 192, 224, 256])
    ap.add_argument("--batches", type=int, nargs="+", default=[1, 2, 4, 8, 16, 32, 64, 96, 128, 192])
    a = ap.parse_args(argv)
    import sys
    sys.path.insert(0, os.path.join(os.path.dirname(os.path.abspath(__file__)), ".."))
    import workloads as wl
    cfg = wl.config(a.config)
    blob = wl.make_weights(cfg.net, cfg.weight_seed, cfg.precision)
    curve = measure_curve(cfg.net, blob, cfg.precision, a.bin_sizes, a.batches, cfg.halo)
    doc = {"what": "rh_enhance kernel time (ms, median of 5) on b bins of S x S pixels, one MI355X",
           "net": f"{cfg.net.topology}{cfg.net.channels} x{cfg.net.scale} blocks={cfg.net.n_blocks} {cfg.precision}",
           "command": "python -m paper_2407_16990_amd.planner --measure OUT.json",
           "curve": {str(S): pts for S, pts in curve.items()}}
    with open(a.measure, "w") as f:
        json.dump(doc, f, indent=1)
    print(json.dumps(doc))
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
