"""ctypes binding of librh.so.  Argument marshalling only: every step of the path runs in the
library's HIP kernels.  torch supplies device memory and the stream.  There is no fallback:
if the library is missing or a call fails, an exception is raised."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))

RH_FP32, RH_BF16 = 0, 1
TOPOLOGY = {"plain": 0, "res": 1, "edsr": 2}
MODE = {"topk": 0, "threshold": 1}
STATUS = ["RH_OK", "RH_E_INVALID", "RH_E_SHAPE", "RH_E_CAPACITY", "RH_E_DEVICE", "RH_E_NOMEM", "RH_E_STATE",
          "RH_E_UNIMPLEMENTED"]

PROF_CLASSES = ["select", "plan", "gather", "head", "conv", "conv_last", "unpack", "temporal"]
PROF_N = len(PROF_CLASSES)

BOX_DTYPE = np.dtype([("frame", "<u4"), ("mbx0", "<u2"), ("mby0", "<u2"), ("wmb", "u1"), ("hmb", "u1"),
                      ("rot", "u1"), ("pad0", "u1"), ("bin", "<u2"), ("bx", "<u2"), ("by", "<u2"),
                      ("pad1", "<u2"), ("id", "<u4")])
PLACE_DTYPE = np.dtype([("mb_id", "<u4"), ("box", "<u4"), ("bin", "<u2"), ("px", "<u2"), ("py", "<u2"),
                        ("rot", "<u2")])
assert BOX_DTYPE.itemsize == 24 and PLACE_DTYPE.itemsize == 16


class NetDesc(C.Structure):
    _fields_ = [("topology", C.c_int32), ("channels", C.c_int32), ("n_blocks", C.c_int32), ("scale", C.c_int32)]


class Config(C.Structure):
    _fields_ = [("frame_w", C.c_int32), ("frame_h", C.c_int32), ("max_frames", C.c_int32), ("halo", C.c_int32),
                ("bin_size", C.c_int32), ("max_bins", C.c_int32), ("connectivity", C.c_int32),
                ("max_box_mbs", C.c_int32), ("precision", C.c_int32), ("net", NetDesc),
                ("sort_policy", C.c_int32), ("rotate", C.c_int32), ("per_layer_tail", C.c_int32)]


class Segment(C.Structure):
    _fields_ = [("frame_begin", C.c_uint32), ("frame_end", C.c_uint32), ("k", C.c_uint32), ("thr", C.c_float)]


class RhError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"{STATUS[status] if 0 <= status < len(STATUS) else status}: {msg}")
        self.status = status


def lib_path() -> str:
    return os.path.join(_HERE, "librh.so")


_lib = None


def _library_is_stale(path: str) -> bool:
    """True when librh.so is missing or was built from other sources than the ones in the tree
    (build.py records a digest of csrc/ and include/ beside the library)."""
    from . import build as _b
    if not os.path.exists(path) or not os.path.exists(_b.STAMP):
        return True
    with open(_b.STAMP) as f:
        return f.read().strip() != _b.source_digest()


def load_library():
    """Load librh.so; it is built first when it is missing or a source file is newer than it."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if _library_is_stale(path):
        from . import build as _b
        _b.build()
    L = C.CDLL(path)
    vp, i32 = C.c_void_p, C.c_int32
    L.rh_budget.restype = C.c_uint32
    L.rh_budget.argtypes = [C.c_uint32] * 3
    L.rh_create.argtypes = [C.POINTER(Config), vp, C.c_size_t, vp, C.POINTER(vp)]
    L.rh_destroy.argtypes = [vp]
    L.rh_destroy.restype = None
    L.rh_set_stream.argtypes = [vp, vp]
    L.rh_last_error.argtypes = [vp]
    L.rh_last_error.restype = C.c_char_p
    L.rh_select_regions.argtypes = [vp, vp, i32, C.POINTER(Segment), i32, i32, vp, vp, vp]
    L.rh_pack.argtypes = [vp, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp]
    L.rh_enhance.argtypes = [vp, vp, i32, i32, i32, vp, vp]
    L.rh_enhance_exact.argtypes = [vp, vp, i32, vp, vp, vp, vp]
    L.rh_enhance_masked.argtypes = [vp, vp, i32, vp, vp, vp, vp]
    L.rh_enhance_needed.argtypes = [vp, vp, i32, vp, vp, vp, vp]
    L.rh_needed_radii.argtypes = [C.POINTER(NetDesc), i32, C.POINTER(i32), i32]
    L.rh_needed_radii.restype = i32
    L.rh_unpack.argtypes = [vp, vp, i32, i32, i32, vp, vp, vp, i32, vp, vp]
    L.rh_identity_places.argtypes = [vp, i32, vp, vp]
    L.rh_read_counts.argtypes = [vp, vp, C.POINTER(C.c_uint32 * 4)]
    L.rh_temporal_phi.argtypes = [vp, vp, i32, i32, i32, vp]
    L.rh_temporal_select.argtypes = [vp, vp, C.POINTER(i32), i32, i32, vp, vp, vp, vp]
    L.rh_temporal_spread.argtypes = [vp, vp, i32, vp, vp]
    L.rh_profile_enable.argtypes = [vp, i32]
    L.rh_profile_read.argtypes = [vp, C.POINTER(C.c_double * PROF_N), C.POINTER(C.c_uint32 * PROF_N)]
    L.rh_select_regions_noalloc.argtypes = [vp, i32, i32, i32, C.POINTER(Segment), i32, i32, vp, vp, vp, vp]
    _lib = L
    return L


NOALLOC_MAX_FRAMES = 4096      # RH_NOALLOC_MAX_FRAMES of include/rh_noalloc.h


def _segments(segments):
    segs = (Segment * max(len(segments), 1))()
    for i, s in enumerate(segments):
        segs[i] = Segment(int(s[0]), int(s[1]), int(s[2]), float(s[3]) if len(s) > 3 else 0.0)
    return segs


def needed_radii(net, per_layer_tail: bool = False):
    """rh_needed_radii: [radius of the first conv, of each conv after it ..., 0 for the tail], or None
    when the needed-region mode does not cover the network."""
    L = load_library()
    out = (C.c_int32 * 512)()
    nb = L.rh_needed_radii(C.byref(NetDesc(TOPOLOGY[net.topology], net.channels, net.n_blocks, net.scale)),
                           1 if per_layer_tail else 0, out, 512)
    return None if nb < 0 else [int(out[i]) for i in range(nb + 2)]


def select_regions_noalloc(importance: torch.Tensor, segments, mask: torch.Tensor, lst: torch.Tensor,
                           n_sel: torch.Tensor, mode="topk", stream=None) -> None:
    """rh_select_regions_noalloc: the selection without a context and without any allocation; the
    caller passes every output (mask u8 [F,MBH,MBW], lst int32 [F*MBH*MBW], n_sel int32 [1])."""
    L = load_library()
    F, mbh, mbw = importance.shape
    assert importance.is_cuda and importance.dtype == torch.float32 and importance.is_contiguous()
    assert mask.is_cuda and mask.numel() >= importance.numel() and lst.numel() >= importance.numel() and n_sel.numel() >= 1
    stream = stream if stream is not None else torch.cuda.current_stream(importance.device)
    st = L.rh_select_regions_noalloc(_ptr(importance), F, mbh, mbw, _segments(segments), len(segments), MODE[mode],
                                     _ptr(mask), _ptr(lst), _ptr(n_sel), C.c_void_p(stream.cuda_stream))
    if st != 0:
        raise RhError(st, "rh_select_regions_noalloc failed (see include/rh_noalloc.h)")


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


@dataclass
class PackOut:
    bins: torch.Tensor
    boxes: torch.Tensor     # u8 [cap, 24]; view with BOX_DTYPE on the host
    places: torch.Tensor    # u8 [cap, 16]
    counts: torch.Tensor    # u32-as-int32 [4]: n_boxes, n_bins, overflow, n_selected


class RH:
    """One context = one configuration on the current device and torch stream."""

    def __init__(self, *, frame_w, frame_h, max_frames, halo, bin_size, max_bins, net, weights: np.ndarray,
                 precision="bf16", connectivity=8, max_box_mbs=0, sort_policy="density", rotate=False,
                 per_layer_tail=False, device="cuda:0", stream=None):
        self.lib = load_library()
        if not torch.cuda.is_available():
            raise RuntimeError("paper_2407_16990_amd needs a GPU: there is no CPU fallback")
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.cfg = Config(frame_w, frame_h, max_frames, halo, bin_size, max_bins, connectivity, max_box_mbs,
                          {"fp32": RH_FP32, "bf16": RH_BF16}[precision],
                          NetDesc(TOPOLOGY[net.topology], net.channels, net.n_blocks, net.scale),
                          {"density": 0, "area": 1}[sort_policy], int(bool(rotate)), int(bool(per_layer_tail)))
        self.scale = net.scale
        self.mbw, self.mbh = (frame_w + 15) // 16, (frame_h + 15) // 16
        w = np.ascontiguousarray(weights, dtype=np.float32)
        self._stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        h = C.c_void_p()
        st = self.lib.rh_create(C.byref(self.cfg), w.ctypes.data_as(C.c_void_p), w.size,
                                C.c_void_p(self._stream.cuda_stream), C.byref(h))
        if st != 0:
            raise RhError(st, "rh_create failed (see include/rh.h for the limits)")
        self.h = h

    def close(self):
        if getattr(self, "h", None):
            self.lib.rh_destroy(self.h)
            self.h = None

    __del__ = close

    def _check(self, st):
        if st != 0:
            raise RhError(st, self.lib.rh_last_error(self.h).decode())

    def budget(self, n_bins: int) -> int:
        return int(self.lib.rh_budget(self.cfg.bin_size, self.cfg.bin_size, n_bins))

    # -- the four calls -------------------------------------------------------------------
    def select_regions(self, importance: torch.Tensor, segments, mode="topk"):
        """importance: cuda f32 [F,MBH,MBW]; segments: rows (frame_begin, frame_end, k[, thr])."""
        F = importance.shape[0]
        assert importance.is_cuda and importance.dtype == torch.float32 and importance.is_contiguous()
        segs = _segments(segments)
        n = importance.numel()
        mask = torch.empty((F, self.mbh, self.mbw), dtype=torch.uint8, device=self.device)
        lst = torch.empty(n, dtype=torch.int32, device=self.device)
        n_sel = torch.empty(1, dtype=torch.int32, device=self.device)
        self._check(self.lib.rh_select_regions(self.h, _ptr(importance), F, segs, len(segments), MODE[mode],
                                               _ptr(mask), _ptr(lst), _ptr(n_sel)))
        return mask, lst, n_sel

    def pack(self, frames: torch.Tensor, importance, mask, lst, n_sel, out: PackOut | None = None) -> PackOut:
        F = frames.shape[0]
        assert frames.is_cuda and frames.dtype == torch.uint8 and frames.is_contiguous()
        S, cap = self.cfg.bin_size, F * self.mbh * self.mbw
        if out is None:
            out = PackOut(torch.empty((self.cfg.max_bins, S, S, 3), dtype=torch.uint8, device=self.device),
                          torch.zeros((cap, 24), dtype=torch.uint8, device=self.device),
                          torch.zeros((cap, 16), dtype=torch.uint8, device=self.device),
                          torch.zeros(4, dtype=torch.int32, device=self.device))
        self._check(self.lib.rh_pack(self.h, _ptr(frames), F, _ptr(importance), _ptr(mask), _ptr(lst), _ptr(n_sel),
                                     _ptr(out.bins), _ptr(out.boxes), _ptr(out.places), _ptr(out.counts)))
        return out

    def enhance(self, imgs: torch.Tensor, n: int | None = None, n_valid: torch.Tensor | None = None,
                out: torch.Tensor | None = None) -> torch.Tensor:
        """imgs: cuda u8 [N,H,W,3] -> raw network output f32 [N,sH,sW,3] (first n images)."""
        assert imgs.is_cuda and imgs.dtype == torch.uint8 and imgs.is_contiguous()
        N, H, W, _ = imgs.shape
        if n is not None:
            N = n
        s = self.scale
        if out is None:
            out = torch.empty((N, H * s, W * s, 3), dtype=torch.float32, device=self.device)
        self._check(self.lib.rh_enhance(self.h, _ptr(imgs), N, H, W, _ptr(out), _ptr(n_valid)))
        return out

    def enhance_exact(self, bins: torch.Tensor, boxes: torch.Tensor, counts: torch.Tensor, n: int | None = None,
                      n_valid: torch.Tensor | None = None, out: torch.Tensor | None = None) -> torch.Tensor:
        """Exact-border variant of enhance for packed bins (boxes, counts as returned by pack)."""
        assert bins.is_cuda and bins.dtype == torch.uint8 and bins.is_contiguous()
        N, H, W, _ = bins.shape
        assert H == W == self.cfg.bin_size
        if n is not None:
            N = n
        s = self.scale
        if out is None:
            out = torch.empty((N, H * s, W * s, 3), dtype=torch.float32, device=self.device)
        self._check(self.lib.rh_enhance_exact(self.h, _ptr(bins), N, _ptr(boxes), _ptr(counts), _ptr(out), _ptr(n_valid)))
        return out

    def enhance_masked(self, bins: torch.Tensor, boxes: torch.Tensor, counts: torch.Tensor, n: int | None = None,
                       n_valid: torch.Tensor | None = None, out: torch.Tensor | None = None) -> torch.Tensor:
        """Box-masked variant of enhance for packed bins (boxes, counts as returned by pack): the body
        convs skip the 8 x 32 cells that no box touches."""
        assert bins.is_cuda and bins.dtype == torch.uint8 and bins.is_contiguous()
        N, H, W, _ = bins.shape
        assert H == W == self.cfg.bin_size
        if n is not None:
            N = n
        s = self.scale
        if out is None:
            out = torch.empty((N, H * s, W * s, 3), dtype=torch.float32, device=self.device)
        self._check(self.lib.rh_enhance_masked(self.h, _ptr(bins), N, _ptr(boxes), _ptr(counts), _ptr(out), _ptr(n_valid)))
        return out

    def enhance_needed(self, bins: torch.Tensor, places: torch.Tensor, counts: torch.Tensor, n: int | None = None,
                       n_valid: torch.Tensor | None = None, out: torch.Tensor | None = None) -> torch.Tensor:
        """Needed-region variant of enhance for packed bins (places, counts as returned by pack): every
        layer computes only the cells that can reach a pasted pixel; the output is defined on the
        pixels of the placed macroblocks only, where it equals enhance's bit for bit."""
        assert bins.is_cuda and bins.dtype == torch.uint8 and bins.is_contiguous()
        N, H, W, _ = bins.shape
        assert H == W == self.cfg.bin_size
        if n is not None:
            N = n
        s = self.scale
        if out is None:
            out = torch.zeros((N, H * s, W * s, 3), dtype=torch.float32, device=self.device)
        self._check(self.lib.rh_enhance_needed(self.h, _ptr(bins), N, _ptr(places), _ptr(counts), _ptr(out), _ptr(n_valid)))
        return out

    def unpack(self, enhanced: torch.Tensor, places, n_places, frames_lr: torch.Tensor, want_sel=False,
               out: torch.Tensor | None = None, sel: torch.Tensor | None = None):
        F, H, W, _ = frames_lr.shape
        s = self.scale
        n_img, oh, ow, _ = enhanced.shape
        if out is None:
            out = torch.empty((F, H * s, W * s, 3), dtype=torch.uint8, device=self.device)
        if want_sel and sel is None:
            sel = torch.zeros((places.shape[0], 16 * s, 16 * s, 3), dtype=torch.float32, device=self.device)
        self._check(self.lib.rh_unpack(self.h, _ptr(enhanced), n_img, oh // s, ow // s, _ptr(places), _ptr(n_places),
                                       _ptr(frames_lr), F, _ptr(out), _ptr(sel)))
        return out, sel

    def identity_places(self, F: int):
        cap = F * self.mbh * self.mbw
        places = torch.zeros((cap, 16), dtype=torch.uint8, device=self.device)
        n = torch.zeros(1, dtype=torch.int32, device=self.device)
        self._check(self.lib.rh_identity_places(self.h, F, _ptr(places), _ptr(n)))
        return places, n

    def temporal_phi(self, res_y: torch.Tensor, tau: int, min_area: int = 1, out: torch.Tensor | None = None):
        """res_y int16 [F,H,W] -> Phi in units of 2^-32, int64 [F] (the bits of the library's uint64)."""
        assert res_y.dtype == torch.int16 and res_y.is_contiguous()
        F = res_y.shape[0]
        assert tuple(res_y.shape[1:]) == (self.cfg.frame_h, self.cfg.frame_w)
        if out is None:
            out = torch.empty(F, dtype=torch.int64, device=self.device)
        self._check(self.lib.rh_temporal_phi(self.h, _ptr(res_y), F, int(tau), int(min_area), _ptr(out)))
        return out

    def temporal_select(self, phi: torch.Tensor, stream_off, n_total: int):
        """-> (alloc int32 [n_streams], selected u8 [F], reuse_from int32 [F], n_selected int32 [1])."""
        ns = len(stream_off) - 1
        off = (C.c_int32 * (ns + 1))(*[int(v) for v in stream_off])
        F = phi.shape[0]
        alloc = torch.zeros(max(ns, 1), dtype=torch.int32, device=self.device)
        selected = torch.zeros(F, dtype=torch.uint8, device=self.device)
        reuse = torch.zeros(F, dtype=torch.int32, device=self.device)
        n_sel = torch.zeros(1, dtype=torch.int32, device=self.device)
        self._check(self.lib.rh_temporal_select(self.h, _ptr(phi), off, ns, int(n_total), _ptr(alloc), _ptr(selected),
                                                _ptr(reuse), _ptr(n_sel)))
        return alloc, selected, reuse, n_sel

    def temporal_spread(self, importance: torch.Tensor, selected: torch.Tensor, reuse_from: torch.Tensor):
        """In place: frames that are not predicted take the map of the frame they reuse."""
        assert importance.dtype == torch.float32 and importance.is_contiguous()
        self._check(self.lib.rh_temporal_spread(self.h, _ptr(importance), importance.shape[0], _ptr(selected), _ptr(reuse_from)))
        return importance

    def read_counts(self, counts: torch.Tensor):
        out = (C.c_uint32 * 4)()
        self._check(self.lib.rh_read_counts(self.h, _ptr(counts), C.byref(out)))
        return list(out)

    def profile_enable(self, on: bool):
        self._check(self.lib.rh_profile_enable(self.h, int(on)))

    def profile_read(self):
        """-> {class: (total ms, launches)} since the last read (synchronises)."""
        ms, n = (C.c_double * PROF_N)(), (C.c_uint32 * PROF_N)()
        self._check(self.lib.rh_profile_read(self.h, C.byref(ms), C.byref(n)))
        return {k: (ms[i], n[i]) for i, k in enumerate(PROF_CLASSES)}

    # host-side views of the metadata
    @staticmethod
    def boxes_np(boxes: torch.Tensor, n: int) -> np.ndarray:
        return boxes[:n].cpu().numpy().view(BOX_DTYPE).reshape(-1)

    @staticmethod
    def places_np(places: torch.Tensor, n: int) -> np.ndarray:
        return places[:n].cpu().numpy().view(PLACE_DTYPE).reshape(-1)
