"""Python face of the CPU oracle (oracle/rh_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the bench's
cpu_baseline leg.  Nothing here touches the HIP library, and the HIP path must
never import this package.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rh_oracle.c")
_LIB = os.path.join(_HERE, "librh_oracle.so")

TOPOLOGY = {"plain": 0, "res": 1, "edsr": 2}


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP across images only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-Wall", "-fopenmp", "-ffp-contract=off",
             "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_budget.restype = C.c_long
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def budget(bin_h: int, bin_w: int, n_bins: int) -> int:
    return int(lib().orc_budget(bin_h, bin_w, n_bins))


def select(imp: np.ndarray, segs: np.ndarray, mode: str = "topk", thr: np.ndarray | None = None):
    """-> (mask u8 [F,mbh,mbw], list u32 [n_sel])."""
    imp = np.ascontiguousarray(imp, dtype=np.float32)
    F, mbh, mbw = imp.shape
    segs = np.ascontiguousarray(segs, dtype=np.uint32).reshape(-1, 3)
    if thr is None:
        thr = np.zeros(len(segs), dtype=np.float32)
    thr = np.ascontiguousarray(thr, dtype=np.float32)
    mask = np.zeros((F, mbh, mbw), dtype=np.uint8)
    lst = np.zeros(max(imp.size, 1), dtype=np.uint32)
    n = C.c_uint32(0)
    rc = lib().orc_select(_p(imp), F, mbh, mbw, _p(segs), _p(thr), len(segs),
                          {"topk": 0, "threshold": 1}[mode], _p(mask), _p(lst), C.byref(n))
    if rc != 0:
        raise ValueError("malformed segments")
    return mask, lst[: n.value].copy()


@dataclass
class Plan:
    boxes: np.ndarray    # int32 [n_boxes, 10]: frame, mbx0, mby0, wmb, hmb, rot, bin, bx, by, id
    places: np.ndarray   # int32 [k, 5]: mb_id, box, bin, px, py
    n_bins: int
    overflow: bool
    place_rot: np.ndarray = None   # int32 [k]: 1 where the MB's box was packed turned


def plan(mask: np.ndarray, imp: np.ndarray, halo: int, bin_size: int, conn: int = 8,
         T: int | None = None, max_bins: int = 1 << 15, sort_policy: str = "density",
         rotate: bool = False) -> Plan:
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    imp = np.ascontiguousarray(imp, dtype=np.float32)
    F, mbh, mbw = mask.shape
    if T is None:
        T = (bin_size - 2 * halo) // 16
    k = int(mask.sum())
    boxes = np.zeros((max(k, 1), 10), dtype=np.int32)
    places = np.zeros((max(k, 1), 5), dtype=np.int32)
    counts = np.zeros(3, dtype=np.int32)
    rots = np.zeros(max(k, 1), dtype=np.int32)
    rc = lib().orc_plan(_p(mask), _p(imp), F, mbh, mbw, halo, bin_size, conn, T, max_bins,
                        {"density": 0, "area": 1}[sort_policy], int(rotate),
                        _p(boxes), _p(places), _p(rots), _p(counts))
    if rc != 0:
        raise ValueError("invalid packing geometry")
    return Plan(boxes[: counts[0]].copy(), places[:k].copy(), int(counts[1]), bool(counts[2]), rots[:k].copy())


def gather(frames: np.ndarray, boxes: np.ndarray, halo: int, bin_size: int, n_bins: int) -> np.ndarray:
    frames = np.ascontiguousarray(frames, dtype=np.uint8)
    F, H, W, _ = frames.shape
    boxes = np.ascontiguousarray(boxes, dtype=np.int32).reshape(-1, 10)
    bins = np.zeros((n_bins, bin_size, bin_size, 3), dtype=np.uint8)
    lib().orc_gather(_p(frames), F, H, W, _p(boxes), len(boxes), halo, bin_size, n_bins, _p(bins))
    return bins


def bilinear(img: np.ndarray, s: int) -> np.ndarray:
    img = np.ascontiguousarray(img, dtype=np.uint8)
    H, W, _ = img.shape
    out = np.zeros((H * s, W * s, 3), dtype=np.uint8)
    lib().orc_bilinear(_p(img), H, W, s, _p(out))
    return out


def conv3x3(x: np.ndarray, w: np.ndarray, b: np.ndarray, relu: bool = False) -> np.ndarray:
    """x fp64 [H,W,Cin]; w fp32 [Cout,3,3,Cin]; b fp32 [Cout] -> fp64 [H,W,Cout]."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    w = np.ascontiguousarray(w, dtype=np.float32)
    b = np.ascontiguousarray(b, dtype=np.float32)
    H, W, Cin = x.shape
    Cout = w.shape[0]
    out = np.zeros((H, W, Cout), dtype=np.float64)
    lib().orc_conv3x3(_p(x), H, W, Cin, _p(w), _p(b), Cout, int(relu), _p(out))
    return out


def pixel_shuffle(x: np.ndarray, r: int) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float64)
    H, W, Cc = x.shape
    out = np.zeros((H * r, W * r, Cc // (r * r)), dtype=np.float64)
    lib().orc_pixel_shuffle(_p(x), H, W, Cc, r, _p(out))
    return out


def border_keep(frame_h: int, frame_w: int, boxes: np.ndarray, halo: int, bin_size: int, n_bins: int) -> np.ndarray:
    """Exact-border mode: u8 [n_bins,S,S], 0 at box pixels whose source lies outside the frame."""
    boxes = np.ascontiguousarray(boxes, dtype=np.int32).reshape(-1, 10)
    keep = np.ones((n_bins, bin_size, bin_size), dtype=np.uint8)
    lib().orc_border_keep(frame_h, frame_w, _p(boxes), len(boxes), halo, bin_size, n_bins, _p(keep))
    return keep


def cell_keep(boxes: np.ndarray, halo: int, bin_size: int, n_bins: int, cell_h: int = 8, cell_w: int = 32) -> np.ndarray:
    """Box-masked mode: u8 [n_bins,S,S], 1 in every cell_h x cell_w cell that a placed box touches."""
    boxes = np.ascontiguousarray(boxes, dtype=np.int32).reshape(-1, 10)
    keep = np.zeros((n_bins, bin_size, bin_size), dtype=np.uint8)
    lib().orc_cell_keep(_p(boxes), len(boxes), halo, bin_size, n_bins, cell_h, cell_w, _p(keep))
    return keep


def sr_forward(net, blob: np.ndarray, imgs: np.ndarray, keep: np.ndarray | None = None,
               body_only: bool = False) -> np.ndarray:
    """imgs u8 [N,H,W,3] -> raw network output fp64 [N,sH,sW,3].  keep (u8 [N,H,W], optional):
    exact-border mode, every layer's output is zeroed where keep == 0; with body_only (box-masked
    mode) only the first conv's and the body convs' outputs are, the layers after the body run
    unmasked."""
    imgs = np.ascontiguousarray(imgs, dtype=np.uint8)
    blob = np.ascontiguousarray(blob, dtype=np.float32)
    N, H, W, _ = imgs.shape
    s = net.scale
    out = np.zeros((N, H * s, W * s, 3), dtype=np.float64)
    if keep is not None:
        keep = np.ascontiguousarray(keep, dtype=np.uint8)
        assert keep.shape == (N, H, W)
    if body_only:
        assert keep is not None
        lib().orc_sr_forward_masked(TOPOLOGY[net.topology], net.channels, net.n_blocks, s, _p(blob),
                                    _p(imgs), N, H, W, _p(keep), _p(out))
        return out
    lib().orc_sr_forward(TOPOLOGY[net.topology], net.channels, net.n_blocks, s, _p(blob),
                         _p(imgs), N, H, W, _p(keep) if keep is not None else None, _p(out))
    return out


def unpack(frames_lr: np.ndarray, s: int, net_out: np.ndarray, places: np.ndarray,
           want_sel: bool = True, place_rot: np.ndarray | None = None):
    """-> (frames_hr u8 [F,sH,sW,3], sel fp32 [k,16s,16s,3] or None)."""
    frames_lr = np.ascontiguousarray(frames_lr, dtype=np.uint8)
    net_out = np.ascontiguousarray(net_out, dtype=np.float64)
    places = np.ascontiguousarray(places, dtype=np.int32).reshape(-1, 5)
    F, H, W, _ = frames_lr.shape
    n_img, oh, ow, _ = net_out.shape
    k = len(places)
    hr = np.zeros((F, H * s, W * s, 3), dtype=np.uint8)
    sel = np.zeros((k, 16 * s, 16 * s, 3), dtype=np.float32) if want_sel else None
    if place_rot is not None:
        place_rot = np.ascontiguousarray(place_rot, dtype=np.int32).reshape(-1)
        assert len(place_rot) == k
    lib().orc_unpack(_p(frames_lr), F, H, W, s, _p(net_out), oh // s, ow // s,
                     _p(places), _p(place_rot) if place_rot is not None else None, k, (W + 15) // 16, (H + 15) // 16,
                     _p(hr), _p(sel) if want_sel else None)
    return hr, sel


def identity_places(F: int, mbh: int, mbw: int) -> np.ndarray:
    """Placement rows for the frame-based run: every MB selected, image n = frame n."""
    g = np.arange(F * mbh * mbw, dtype=np.int32)
    f, rem = g // (mbh * mbw), g % (mbh * mbw)
    y, x = rem // mbw, rem % mbw
    return np.stack([g, f, f, 16 * x, 16 * y], axis=1).astype(np.int32)


@dataclass
class PathResult:
    mask: np.ndarray
    list: np.ndarray
    plan: Plan
    bins: np.ndarray
    net_out: np.ndarray
    frames_hr: np.ndarray
    sel: np.ndarray


def run_path(frames, imp, segs, net, blob, halo, bin_size, conn=8, T=None,
             mode="topk", thr=None, max_bins=1 << 15, sort_policy="density", rotate=False,
             exact_border=False, box_masked=False) -> PathResult:
    """The whole hot path: select -> plan -> gather -> SR -> paste."""
    mask, lst = select(imp, segs, mode, thr)
    pl = plan(mask, imp, halo, bin_size, conn, T, max_bins, sort_policy, rotate)
    bins = gather(frames, pl.boxes, halo, bin_size, pl.n_bins)
    keep = border_keep(frames.shape[1], frames.shape[2], pl.boxes, halo, bin_size, pl.n_bins) if exact_border else None
    if box_masked:
        assert not exact_border
        net_out = sr_forward(net, blob, bins, cell_keep(pl.boxes, halo, bin_size, pl.n_bins), body_only=True)
    else:
        net_out = sr_forward(net, blob, bins, keep)
    hr, sel = unpack(frames, net.scale, net_out, pl.places, place_rot=pl.place_rot)
    return PathResult(mask, lst, pl, bins, net_out, hr, sel)
