"""CPU oracle of the temporal importance reuse step (Sec. 3.2.2).

TEST INFRASTRUCTURE ONLY (see the package docstring).  The operator itself (thresholding, blob
labelling, inverse areas) is the C routine orc_phi; everything after it is exact integer
arithmetic on Python ints, written as the definitions read:

  * S_i = |Phi_{i+1} - Phi_i| for the n-1 steps of a stream's chunk, L1-normalised; the
    cumulative distribution gives every frame a position P_f = (S_0 + ... + S_{f-1}) / sum(S)
    in [0, 1], P_0 = 0 (all positions 0 when nothing changed at all);
  * the axis [0, 1] is cut into N equal intervals; frame f lies in interval
    min(N-1, floor(N * P_f)); in every interval that holds a frame, the frame whose position
    is nearest the interval's midpoint (earliest on ties) is the one to be predicted, and the
    other frames of the interval reuse its importance map;
  * with several streams, every stream gets one predicted frame, and the rest of the budget is
    shared in proportion to the streams' total change sum_i S_i (largest remainders, ties to
    the lower stream; equal shares when no stream changed).

The paper gives the normalisation, the equal cuts of the CDF and the proportional share; which
value is taken inside an interval, how the share is rounded, and that no stream may go without
a prediction are readings of this implementation.  No value of these is
printed in the paper: the functions are pinned by closed-form cases in tests/test_oracle_temporal.py.
"""
from __future__ import annotations

import ctypes as C

import numpy as np

from . import lib, _p


def phi(res: np.ndarray, tau: int, min_area: int = 1):
    """res int16 [F,H,W] -> (Phi in units of 2^-32 as uint64 [F], blob counts int32 [F])."""
    res = np.ascontiguousarray(res, dtype=np.int16)
    F, H, W = res.shape
    out = np.zeros(F, dtype=np.uint64)
    nb = np.zeros(F, dtype=np.int32)
    lib().orc_phi(_p(res), F, H, W, int(tau), int(min_area), _p(out), _p(nb))
    return out, nb


def change_totals(phi_q: np.ndarray, stream_off) -> list[int]:
    """Total absolute change of Phi over each stream's chunk."""
    tot = []
    for s in range(len(stream_off) - 1):
        v = [int(x) for x in phi_q[stream_off[s]:stream_off[s + 1]]]
        tot.append(sum(abs(v[i + 1] - v[i]) for i in range(len(v) - 1)))
    return tot


def allocate(totals: list[int], n_total: int) -> list[int]:
    """Frames to predict per stream: one each, the rest in proportion to the totals."""
    ns = len(totals)
    if n_total < ns:
        raise ValueError("the budget must cover one frame per stream")
    rest, whole = n_total - ns, sum(totals)
    if whole == 0:
        return [1 + rest // ns + (1 if s < rest % ns else 0) for s in range(ns)]
    quota = [rest * t // whole for t in totals]
    rem = [rest * t % whole for t in totals]
    left = rest - sum(quota)
    order = sorted(range(ns), key=lambda s: (-rem[s], s))
    for s in order[:left]:
        quota[s] += 1
    return [1 + q for q in quota]


def frame_select(phi_stream: list[int], N: int):
    """One stream's chunk -> (sorted list of frames to predict, reuse_from[f] for every frame)."""
    n = len(phi_stream)
    S = [abs(phi_stream[i + 1] - phi_stream[i]) for i in range(n - 1)]
    T = sum(S)
    A = [sum(S[:f]) for f in range(n)]                     # numerators of the positions P_f = A_f / T
    interval = [min(N - 1, N * A[f] // T) if T else 0 for f in range(n)]
    # distance from the midpoint (2j+1)/(2N), scaled by 2*N*T to stay in integers
    dist = [abs(2 * N * A[f] - (2 * interval[f] + 1) * T) for f in range(n)]
    rep = {}
    for f in range(n):
        j = interval[f]
        if j not in rep or dist[f] < dist[rep[j]]:
            rep[j] = f
    return sorted(rep.values()), [rep[interval[f]] for f in range(n)]


def temporal_plan(phi_q: np.ndarray, stream_off, n_total: int):
    """-> (alloc per stream, selected u8 [F], reuse_from u32 [F] as batch-wide frame indices)."""
    F = len(phi_q)
    alloc = allocate(change_totals(phi_q, stream_off), n_total)
    selected = np.zeros(F, dtype=np.uint8)
    reuse = np.zeros(F, dtype=np.uint32)
    for s in range(len(stream_off) - 1):
        b, e = int(stream_off[s]), int(stream_off[s + 1])
        picks, frm = frame_select([int(x) for x in phi_q[b:e]], alloc[s])
        for f in picks:
            selected[b + f] = 1
        reuse[b:e] = [b + r for r in frm]
    return alloc, selected, reuse


def spread(imp: np.ndarray, reuse_from: np.ndarray) -> np.ndarray:
    """Every frame takes the importance map of the frame it reuses."""
    return np.ascontiguousarray(imp[np.asarray(reuse_from, dtype=np.int64)])
