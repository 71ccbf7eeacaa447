"""Shared helpers of the GPU parity tests: run the HIP path through the C ABI binding and
compare every output with the CPU oracle on the same seeded inputs."""
from __future__ import annotations

import numpy as np
import torch

import oracle
import workloads as wl
from paper_2407_16990_amd import RH


def make_rh(cfg: wl.Config, blob, n_frames=None, max_bins=None, precision=None, **kw) -> RH:
    F = cfg.n_frames if n_frames is None else n_frames
    if max_bins is None:
        max_bins = max(4, F * cfg.mbw * cfg.mbh)          # never overflows
    return RH(frame_w=cfg.width, frame_h=cfg.height, max_frames=F, halo=cfg.halo, bin_size=cfg.bin_size,
              max_bins=min(max_bins, 60000), net=cfg.net, weights=blob,
              precision=precision or cfg.precision, **kw)


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def gpu_select(rh: RH, imp: np.ndarray, segs, mode="topk"):
    mask, lst, n_sel = rh.select_regions(dev(imp), segs, mode)
    n = int(n_sel.cpu()[0])
    return mask.cpu().numpy(), lst[:n].cpu().numpy().astype(np.uint32), (mask, lst, n_sel)


def boxes_as_rows(b: np.ndarray) -> np.ndarray:
    return np.stack([b[k].astype(np.int64) for k in ("frame", "mbx0", "mby0", "wmb", "hmb", "rot", "bin", "bx", "by", "id")], axis=1)


def places_as_rows(p: np.ndarray) -> np.ndarray:
    return np.stack([p[k].astype(np.int64) for k in ("mb_id", "box", "bin", "px", "py")], axis=1)


def check_select_and_plan(rh: RH, cfg, frames, imp, segs, mode="topk", thr=None, conn=8, T=None, max_bins=1 << 15,
                          sort_policy="density", rotate=False):
    """Selection + plan + packed bytes, bit-exact.  Returns (oracle plan, gpu pack output, dev handles)."""
    seg_rows = [tuple(s) + ((float(thr[i]),) if thr is not None else ()) for i, s in enumerate(np.asarray(segs).tolist())]
    o_mask, o_list = oracle.select(imp, np.asarray(segs, dtype=np.uint32).reshape(-1, 3), mode, thr)
    g_mask, g_list, handles = gpu_select(rh, imp, seg_rows, mode)
    assert np.array_equal(g_mask, o_mask), "mask differs"
    assert np.array_equal(g_list, o_list), "list differs"
    o_plan = oracle.plan(o_mask, imp, cfg.halo, cfg.bin_size, conn, T, max_bins, sort_policy, rotate)
    d_frames, d_imp = dev(frames), dev(imp)
    po = rh.pack(d_frames, d_imp, *handles)
    counts = po.counts.cpu().numpy().astype(np.int64)
    assert counts.tolist() == [len(o_plan.boxes), o_plan.n_bins, int(o_plan.overflow), len(o_list)], counts
    g_boxes = boxes_as_rows(RH.boxes_np(po.boxes, counts[0]))
    g_places = places_as_rows(RH.places_np(po.places, counts[3]))
    assert np.array_equal(g_boxes, o_plan.boxes.astype(np.int64)), "boxes differ"
    assert np.array_equal(g_places, o_plan.places.astype(np.int64)), "places differ"
    assert np.array_equal(RH.places_np(po.places, counts[3])["rot"].astype(np.int64), o_plan.place_rot), "turned flags differ"
    o_bins = oracle.gather(frames, o_plan.boxes, cfg.halo, cfg.bin_size, o_plan.n_bins)
    g_bins = po.bins[: o_plan.n_bins].cpu().numpy()
    assert np.array_equal(g_bins, o_bins), "packed bytes differ"
    return o_plan, po, (d_frames, d_imp, o_bins)


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64); b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-30))


# bf16 path, element-wise bars.  The rounding points of the bf16 path (activations stored as bf16
# between layers; with 16 residual blocks the 17 roundings of the residual stream carry two thirds
# of the error variance) put a relative error of about 0.9 % rms on the network output (0.5 % with
# 2 blocks).  An element's error scales with the local activation level, so the distribution has
# heavy tails: over the 20 million pasted values of configuration 3 the extreme is 0.103 x the
# output's rms (measured on all 1632 macroblocks: 8.64e-3 at rms 0.084).  The 2/255 bar on pasted
# pixels therefore holds for network outputs of rms <= 0.07 - the benchmark nets are drawn with
# rms 0.05, a trained SR net's correction to the interpolated frame being a few hundredths - and
# above that the bar grows with the rms.  The raw network output also covers halos, box borders and
# empty bin area (60 million values per batch of configuration 3, activation peaks several times
# the rms): its element-wise bar is 0.15 x rms; a wrong pixel or channel is an error of the order
# of the rms itself.
BF16_RMS_LIMIT = 0.07


def bf16_max_abs_bar(o_net) -> float:
    """Bar on pasted (enhanced, clamped) pixels."""
    rms = float(np.sqrt(np.mean(np.asarray(o_net, dtype=np.float64) ** 2)))
    return 2.0 / 255.0 * max(1.0, rms / BF16_RMS_LIMIT)


def check_net(g_net, o_net, precision, what=""):
    """Raw network output, GPU against oracle: the norm and every element."""
    g = np.asarray(g_net, dtype=np.float64); o = np.asarray(o_net, dtype=np.float64)
    assert g.shape == o.shape
    rms = float(np.sqrt(np.mean(o ** 2)))
    e, worst = rel_l2(g, o), float(np.abs(g - o).max())
    bar = 1e-4 * max(1.0, float(np.abs(o).max())) if precision == "fp32" else max(2.0 / 255.0, 0.15 * rms)
    print(f"[{what}/{precision}] net rel-L2={e:.3e} max abs={worst:.3e} (bar {bar:.3e}, rms {rms:.3f}, max |net| {np.abs(o).max():.3f})", flush=True)
    assert e <= (1e-5 if precision == "fp32" else 1e-2), e
    assert worst <= bar, (worst, bar)
    return e, worst
