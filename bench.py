#!/usr/bin/env python3
"""Benchmark of the region-aware enhancer hot path on one MI355X.

A step = one pass of the whole path (rh_select_regions -> rh_pack -> rh_enhance -> rh_unpack)
over one batch of synthetic input already resident in HBM.  Workload: configuration 3 of the
benchmark list (16 frames 480x272, EDSR-baseline x4, top 20 % macroblocks, halo 10, 128x128
bins, bf16), the one the headline metric "enhanced macroblocks/s" is quoted on.

Prints ONE JSON line with the metric, the roofline of the dominant kernel (the bf16 MFMA conv of
the network body, timed with HIP events on the library's stream inside the timed region), the
CPU oracle timed on a bounded sample (cpu_baseline), the 100 %-macroblock frame-based run, the
memory-bound steps at batch size and on 16 batches, the other benchmark configurations
(other_configs: 1, 2, 5 and the selected-fraction sweep of configuration 4), planner-lite's choice
of the bin size (planner_lite) and the temporal importance reuse leg.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK = 2.5e15    # dense bf16 MFMA, FLOP/s (MI355X published)
FP32_VALU_PEAK = 157.3e12  # fp32 vector ALUs, FLOP/s (MI355X published)
HBM_PEAK = 8.0e12          # B/s
# HBM bytes per launch of the dominant kernel class on the default workload: NOT measured live but
# taken from the rocprofv3 FETCH_SIZE / WRITE_SIZE runs summarised in the named profile (scaled by
# the plain-copy calibration stated there); only reported for that workload and kernel set.
PROFILED_TRAFFIC = {"cfg3_16x480x272_edsr64_x4_bf16": (404.2e6, "profiles/conv_mfma_cfg3_hbm_counters.md")}
CONV_KERNEL = {64: "k_conv_mfma_duo<SKIP,RELU,10> (64-channel bf16-output convs of the network body: ReLU and skip-add instantiations)",
               32: "k_conv_mfma<32,1,16,false,SKIP,RELU> (bf16-output 32-channel convs)"}


def live_cell_fraction(boxes, halo, S, n_bins, cell_h=8, cell_w=32):
    """Share of the bins' cell_h x cell_w cells that a placed box (with its halo) touches: what the
    body convs of the box-masked enhance mode compute."""
    cx, cy = -(-S // cell_w), -(-S // cell_h)
    live = np.zeros((max(n_bins, 1), cy, cx), dtype=bool)
    for b in boxes:
        if int(b["bin"]) >= n_bins:
            continue
        bw, bh = 16 * int(b["wmb"]) + 2 * halo, 16 * int(b["hmb"]) + 2 * halo
        fw, fh = (bh, bw) if int(b["rot"]) else (bw, bh)
        x0, y0 = int(b["bx"]), int(b["by"])
        live[int(b["bin"]), y0 // cell_h:(y0 + fh - 1) // cell_h + 1, x0 // cell_w:(x0 + fw - 1) // cell_w + 1] = True
    return float(live.mean()) if n_bins else 1.0


def needed_cell_fractions(places, S, n_bins, radii, cell_h=8, cell_w=32):
    """Needed-region mode: for every radius, the share of the bins' cells within that Chebyshev distance
    of a placed macroblock (what the layer of that radius computes)."""
    cx, cy = -(-S // cell_w), -(-S // cell_h)
    dmin = np.full((max(n_bins, 1), cy, cx), 1 << 30, dtype=np.int64)
    ys, xs = np.arange(cy) * cell_h, np.arange(cx) * cell_w
    for p in places:
        b, x0, y0 = int(p["bin"]), int(p["px"]), int(p["py"])
        if b >= n_bins:
            continue
        gy = np.maximum(0, np.maximum(ys - (y0 + 15), y0 - (ys + cell_h - 1)))
        gx = np.maximum(0, np.maximum(xs - (x0 + 15), x0 - (xs + cell_w - 1)))
        np.minimum(dmin[b], np.maximum(gy[:, None], gx[None, :]), out=dmin[b])
    return [float((dmin <= r).mean()) for r in radii]


def net_flops(net, composed_tail):
    """Per packed low-resolution pixel: flop and launches of the profiled conv class (bf16 path: the
    C-input / bf16-output convs; 18*cin*cout per output pixel at the layer's resolution), the
    network's flop as defined layer by layer, and the flop the kernels execute (they differ when
    the linear tail of an EDSR-shaped net runs as one composed 5x5 conv on padded MFMA rows)."""
    C, s = net.channels, net.scale
    body = net.n_blocks - 2 if net.topology == "plain" else 2 * net.n_blocks + (1 if net.topology == "edsr" else 0)
    cls_fl, cls_n = body * 18 * C * C, body
    head = 18 * 3 * C
    if net.topology == "edsr":
        ups = 18 * C * 4 * C + 4 * 18 * C * 4 * C if s == 4 else 18 * C * C * s * s
        network = head + cls_fl + ups + s * s * 18 * C * 3
        if composed_tail:
            executed = head + cls_fl + 2 * 25 * C * 32 * (2 if s == 4 else 1)
        else:
            executed = network
            cls_fl += ups
            cls_n += 2 if s == 4 else 1
    else:
        network = executed = head + cls_fl + 18 * C * 3 * s * s
    return cls_fl, cls_n, network, executed


class Runner:
    """One configuration resident on the GPU: inputs, context, preallocated outputs, and a step()."""

    def __init__(self, cfg, args, max_box_mbs=0, per_layer_tail=False):
        import torch
        import workloads as wl
        from paper_2407_16990_amd import RH
        self.torch, self.cfg = torch, cfg
        F, S = cfg.n_frames, cfg.bin_size
        self.frames, self.imp, self.segs = wl.make_frames(cfg), wl.make_importance(cfg), wl.make_segments(cfg)
        self.blob = wl.make_weights(cfg.net, cfg.weight_seed, cfg.precision)
        # room for the packer's worst case (isolated macroblocks: one box each)
        worst = cfg.index == 5 or cfg.importance == "uniform" or max_box_mbs == 1 or cfg.frac > 0.3
        self.max_bins = (512 if worst else 256) * max(1, (128 // S) ** 2)
        self.composed = (cfg.precision == "bf16" and cfg.net.topology == "edsr" and not per_layer_tail
                         and not args.exact_border)
        self.rh = RH(frame_w=cfg.width, frame_h=cfg.height, max_frames=F, halo=cfg.halo, bin_size=S, max_bins=self.max_bins,
                     net=cfg.net, weights=self.blob, precision=cfg.precision, max_box_mbs=max_box_mbs,
                     per_layer_tail=per_layer_tail)
        self.d_frames = torch.from_numpy(self.frames).cuda()
        self.d_imp = torch.from_numpy(self.imp).cuda()
        self.seg_rows = [tuple(r) for r in self.segs.tolist()]
        self.po = None
        self.exact = args.exact_border
        self.masked = bool(getattr(args, "box_masked", False)) and cfg.precision == "bf16" and cfg.net.channels == 64
        self.live_frac = 1.0      # box-masked / needed-region mode: mean fraction of the 8 x 32 cells that the body convs compute
        self.needed = (bool(getattr(args, "needed_region", False)) and cfg.precision == "bf16" and cfg.net.channels == 64
                       and not per_layer_tail)
        self.sync_counts = args.sync_counts
        self.net_out = self.hr = None
        self.cap = 0

    def alloc(self, n_bins_cap):
        torch, cfg = self.torch, self.cfg
        s, S = cfg.net.scale, cfg.bin_size
        self.cap = n_bins_cap
        self.net_out = torch.empty((n_bins_cap, S * s, S * s, 3), dtype=torch.float32, device="cuda")
        self.hr = torch.empty((cfg.n_frames, cfg.height * s, cfg.width * s, 3), dtype=torch.uint8, device="cuda")

    def plan_only(self):
        rh = self.rh
        mask, lst, n_sel = rh.select_regions(self.d_imp, self.seg_rows)
        self.po = rh.pack(self.d_frames, self.d_imp, mask, lst, n_sel, out=self.po)
        return rh.read_counts(self.po.counts)

    def step(self):
        rh = self.rh
        mask, lst, n_sel = rh.select_regions(self.d_imp, self.seg_rows)
        self.po = po = rh.pack(self.d_frames, self.d_imp, mask, lst, n_sel, out=self.po)
        if self.exact:
            rh.enhance_exact(po.bins, po.boxes, po.counts, n=self.cap, n_valid=po.counts[1:2], out=self.net_out)
        elif self.masked:
            rh.enhance_masked(po.bins, po.boxes, po.counts, n=self.cap, n_valid=po.counts[1:2], out=self.net_out)
        elif self.needed:
            rh.enhance_needed(po.bins, po.places, po.counts, n=self.cap, n_valid=po.counts[1:2], out=self.net_out)
        elif self.sync_counts:
            rh.enhance(po.bins, n=rh.read_counts(po.counts)[1], out=self.net_out)
        else:
            rh.enhance(po.bins, n=self.cap, n_valid=po.counts[1:2], out=self.net_out)   # device-side bin count
        rh.unpack(self.net_out, po.places, po.counts[3:4], self.d_frames, out=self.hr)

    def timed(self, steps, warmup):
        """-> (ms per step, per-class kernel (ms, launches) per step, counts)."""
        torch, rh = self.torch, self.rh
        counts = self.plan_only()
        if self.masked:
            self.live_frac = live_cell_fraction(rh.boxes_np(self.po.boxes, counts[0]), self.cfg.halo, self.cfg.bin_size, counts[1])
        if self.needed:
            from paper_2407_16990_amd import needed_radii
            radii = needed_radii(self.cfg.net)
            fr = needed_cell_fractions(rh.places_np(self.po.places, counts[3]), self.cfg.bin_size, counts[1], radii)
            self.live_frac = float(np.mean(fr[1:-1])) if len(fr) > 2 else 1.0
            self.tail_frac = fr[-1]
        if self.net_out is None:
            # all outputs are allocated once, outside the timed region; the enhance call is sized by
            # the output capacity (the bins this batch needs plus slack) and told the device-side count
            self.alloc(min(self.max_bins, counts[1] + 8))
        for _ in range(warmup):
            self.step()
        torch.cuda.synchronize()
        rh.profile_enable(True)
        rh.profile_read()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            self.step()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        prof = rh.profile_read()
        rh.profile_enable(False)
        return dt / steps * 1e3, {k: (v[0] / steps, v[1] / steps) for k, v in prof.items()}, counts

    def frame_based(self, steps):
        """100 % of the macroblocks: rh_enhance on whole frames + identity placement -> ms per step."""
        torch, rh, cfg = self.torch, self.rh, self.cfg
        s, F = cfg.net.scale, cfg.n_frames
        places, n_pl = rh.identity_places(F)
        fb_net = torch.empty((F, cfg.height * s, cfg.width * s, 3), dtype=torch.float32, device="cuda")
        if self.hr is None:
            self.alloc(1)

        def fb_step():
            rh.enhance(self.d_frames, out=fb_net)
            rh.unpack(fb_net, places, n_pl, self.d_frames, out=self.hr)
        fb_step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fb_step()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps * 1e3

    def summary(self, ms, prof, counts):
        cfg = self.cfg
        S = cfg.bin_size
        n_boxes, n_bins, _, k_sel = counts
        px_lr = n_bins * S * S
        cls_fl, cls_n, network_fl, executed_fl = net_flops(cfg.net, self.composed)
        if cfg.precision != "bf16":
            import workloads as wl
            cls_fl, cls_n = network_fl, len(wl.net_layers(cfg.net))      # fp32 path: all layers are one class
        conv_ms, conv_n = prof["conv"]
        launch_s = conv_ms / max(conv_n, 1) * 1e-3
        flop_per_launch = cls_fl * px_lr * self.live_frac / max(cls_n, 1)      # box-masked mode: live cells only
        achieved = flop_per_launch / launch_s if launch_s > 0 else 0.0
        peak = MFMA_BF16_PEAK if cfg.precision == "bf16" else FP32_VALU_PEAK
        enh_s = sum(prof[k][0] for k in ("head", "conv", "conv_last")) * 1e-3
        return {"ms_per_step": ms, "macroblocks_per_s": k_sel / (ms * 1e-3), "n_selected": k_sel, "n_boxes": n_boxes,
                "n_bins": n_bins, "occupy_ratio": 256.0 * k_sel / px_lr if px_lr else 0.0,
                "kernel_ms_per_step": {k: v[0] for k, v in prof.items()},
                "conv_class": {"achieved_tflops": achieved / 1e12, "frac_of_peak": achieved / peak, "avg_launch_us": launch_s * 1e6,
                               "launches_per_step": conv_n, "flop_per_launch": flop_per_launch},
                "enhance_tflops_executed": executed_fl * px_lr / max(enh_s, 1e-12) / 1e12,
                "enhance_tflops_network": network_fl * px_lr / max(enh_s, 1e-12) / 1e12}

    def close(self):
        self.rh.close()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-frame-based", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip configurations 1, 2, 5 and the selected-fraction sweep of configuration 4")
    ap.add_argument("--fraction", type=float, default=None, help="override the selected fraction of the configuration")
    ap.add_argument("--importance", choices=["clustered", "uniform"], default=None,
                    help="override the importance recipe (uniform = iid, isolated macroblocks: the packer's worst case)")
    ap.add_argument("--box-masked", action="store_true",
                    help="enhance with rh_enhance_masked (the body convs skip the 8 x 32 cells that no box touches; "
                         "a different function near those cells)")
    ap.add_argument("--no-box-masked-leg", action="store_true", help="skip the box-masked leg of the default run")
    ap.add_argument("--needed-region", action="store_true",
                    help="enhance with rh_enhance_needed (every layer computes only the cells that can reach a pasted "
                         "pixel; pasted pixels bit-identical to rh_enhance)")
    ap.add_argument("--no-needed-region-leg", action="store_true", help="skip the needed-region leg of the default run")
    ap.add_argument("--exact-border", action="store_true",
                    help="enhance with rh_enhance_exact (per-layer zeroing of the out-of-frame part of the boxes)")
    ap.add_argument("--per-layer-tail", action="store_true",
                    help="run the upsampler and the last conv layer by layer instead of as one composed convolution")
    ap.add_argument("--bin-size", type=int, default=None, help="override the bin side S (pixels)")
    ap.add_argument("--max-box-mbs", type=int, default=0,
                    help="Partition's preset size in macroblocks (0 = the largest that fits a bin; 1 = every "
                         "macroblock its own box, the paper's MB-packing / Block policy)")
    ap.add_argument("--mem-batch", type=int, default=16, metavar="X",
                    help="also time the memory-bound steps (pack gather, unpack) on X copies of the batch, where "
                         "they are large enough to be bandwidth- rather than launch-bound (0 = skip)")
    ap.add_argument("--no-temporal", action="store_true",
                    help="skip the temporal importance reuse leg (Sec. 3.2.2; reported beside the path, not in `value`)")
    ap.add_argument("--no-planner", action="store_true", help="skip planner-lite's choice of the bin size")
    ap.add_argument("--temporal-streams", type=int, default=10, help="streams of the temporal leg's chunk")
    ap.add_argument("--temporal-frames", type=int, default=30, help="frames per stream of the temporal leg's chunk")
    ap.add_argument("--sync-counts", action="store_true",
                    help="read the bin count back to the host after rh_pack (one synchronisation per step) and "
                         "enhance exactly that many bins, instead of passing the device-side count")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (--gpus 1); no multi-GPU figure exists", file=sys.stderr)
        sys.exit(2)

    import torch
    import workloads as wl
    from paper_2407_16990_amd import RH

    cfg = wl.config(args.config)
    if args.fraction is not None:
        cfg = wl.replace(cfg, frac=args.fraction, name=f"{cfg.name}_frac{args.fraction:g}")
    if args.importance is not None and args.importance != cfg.importance:
        cfg = wl.replace(cfg, importance=args.importance, name=f"{cfg.name}_{args.importance}")
    if args.bin_size is not None and args.bin_size != cfg.bin_size:
        cfg = wl.replace(cfg, bin_size=args.bin_size, name=f"{cfg.name}_S{args.bin_size}")
    if args.max_box_mbs:
        cfg = wl.replace(cfg, name=f"{cfg.name}_T{args.max_box_mbs}")
    if args.exact_border:
        cfg = wl.replace(cfg, name=f"{cfg.name}_exact_border")
    if args.per_layer_tail:
        cfg = wl.replace(cfg, name=f"{cfg.name}_per_layer_tail")
    if args.box_masked:
        cfg = wl.replace(cfg, name=f"{cfg.name}_box_masked")
    if args.needed_region:
        cfg = wl.replace(cfg, name=f"{cfg.name}_needed_region")
    F, s, S = cfg.n_frames, cfg.net.scale, cfg.bin_size

    # A plain device copy of known size, outside every timed region: what rocprofv3's FETCH_SIZE /
    # WRITE_SIZE read for it calibrates those counters in a counter run of this same command.
    cal_src = torch.full((256 << 20,), 7, dtype=torch.uint8, device="cuda")
    cal_dst = torch.empty_like(cal_src)
    cal_dst.copy_(cal_src)
    torch.cuda.synchronize()
    del cal_src, cal_dst

    run = Runner(cfg, args, max_box_mbs=args.max_box_mbs, per_layer_tail=args.per_layer_tail)
    ms_step, prof, counts = run.timed(args.steps, args.warmup)
    sm = run.summary(ms_step, prof, counts)
    n_boxes, n_bins, _, k_sel = counts
    rh, po, d_frames, d_imp, seg_rows, blob = run.rh, run.po, run.d_frames, run.d_imp, run.seg_rows, run.blob
    frames, imp, segs = run.frames, run.imp, run.segs
    px_lr = n_bins * S * S
    cc = sm["conv_class"]
    traffic = PROFILED_TRAFFIC.get(cfg.name) if run.composed else None

    result = {
        "metric": "enhanced macroblocks/s",
        "value": sm["macroblocks_per_s"], "unit": "MB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.precision == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": cfg.name, "frames": F, "frame": [cfg.width, cfg.height], "scale": s,
                   "selected_fraction": cfg.frac, "halo": cfg.halo, "bin_size": S,
                   "n_selected": k_sel, "n_boxes": n_boxes, "n_bins": n_bins, "occupy_ratio": sm["occupy_ratio"],
                   "tail": "composed 5x5 conv" if run.composed else "layer by layer"},
        "output_mpixel_per_s": F * cfg.height * s * cfg.width * s / (ms_step * 1e-3) / 1e6,
        "kernel_ms_per_step": sm["kernel_ms_per_step"],
        "roofline": {"bound": "mfma" if cfg.precision == "bf16" else "alu",
                     "kernel": CONV_KERNEL.get(cfg.net.channels, "k_conv_mfma") if cfg.precision == "bf16" else "k_conv3x3_f32 (all layers)",
                     "achieved": cc["achieved_tflops"], "peak": (MFMA_BF16_PEAK if cfg.precision == "bf16" else FP32_VALU_PEAK) / 1e12,
                     "unit": "TFLOP/s", "frac": cc["frac_of_peak"],
                     "traffic": traffic[0] if traffic else None, "traffic_source": traffic[1] if traffic else None,
                     "avg_launch_us": cc["avg_launch_us"], "launches_per_step": cc["launches_per_step"],
                     "flop_per_launch": cc["flop_per_launch"]},
        "enhance_tflops_executed": sm["enhance_tflops_executed"],
        "enhance_tflops_network": sm["enhance_tflops_network"],
    }

    # ---- the memory-bound steps: algorithmic bytes / event time, at batch size and at X batches ----
    def mem_bytes(nb, boxes_host, nsel, nf):
        box_px = sum((16 * int(b["wmb"]) + 2 * cfg.halo) * (16 * int(b["hmb"]) + 2 * cfg.halo) for b in boxes_host)
        pack_b = nb * S * S * 3 + box_px * 3                      # every bin byte written, box pixels read
        unpack_b = nf * cfg.height * s * cfg.width * s * 3 + nf * cfg.height * cfg.width * 3 + nsel * (16 * s) ** 2 * 3 * 4
        return pack_b, unpack_b

    def mem_row(nbytes, ms):
        us = ms * 1e3
        gbs = nbytes / (us * 1e-6) / 1e9 if us > 0 else 0.0
        return {"bytes": nbytes, "us": us, "GB/s": gbs, "frac_of_hbm_peak": gbs * 1e9 / HBM_PEAK}

    boxes_host = RH.boxes_np(po.boxes, n_boxes)
    pb, ub = mem_bytes(n_bins, boxes_host, k_sel, F)
    sel_bytes = lambda nf, nsel: nf * rh.mbh * rh.mbw * 5 + nsel * 4          # 4 B read + 1 B mask per MB, 4 B per selected MB
    result["memory_steps"] = {
        "select": dict(mem_row(sel_bytes(F, k_sel), prof["select"][0]), note="latency-bound: tens of kilobytes"),
        "plan": {"us": prof["plan"][0] * 1e3,
                 "share_of_enhance_time": prof["plan"][0] / max(prof["head"][0] + prof["conv"][0] + prof["conv_last"][0], 1e-12)},
        "pack_gather": mem_row(pb, prof["gather"][0]),
        "unpack": mem_row(ub, prof["unpack"][0]),
        "hbm_peak_GB/s": HBM_PEAK / 1e9}
    if args.mem_batch > 0:
        X = args.mem_batch
        rhx = RH(frame_w=cfg.width, frame_h=cfg.height, max_frames=F * X, halo=cfg.halo, bin_size=cfg.bin_size,
                 max_bins=run.max_bins * X, net=cfg.net, weights=blob, precision=cfg.precision,
                 max_box_mbs=args.max_box_mbs)
        xf = d_frames.repeat(X, 1, 1, 1)
        xi = d_imp.repeat(X, 1, 1)
        xsegs = [(r[0] + j * F, r[1] + j * F) + tuple(r[2:]) for j in range(X) for r in seg_rows]
        xhr = torch.empty((F * X, cfg.height * s, cfg.width * s, 3), dtype=torch.uint8, device="cuda")
        xpo = None
        xnet = None
        reps = 5
        for it in range(reps + 1):
            if it == 1:
                rhx.profile_enable(True)
                rhx.profile_read()
            m_, l_, n_ = rhx.select_regions(xi, xsegs)
            xpo = rhx.pack(xf, xi, m_, l_, n_, out=xpo)
            if xnet is None:
                xc = rhx.read_counts(xpo.counts)
                # unpack only reads the enhanced tensor: any values do for timing
                xnet = torch.zeros((xc[1], S * s, S * s, 3), dtype=torch.float32, device="cuda")
            rhx.unpack(xnet, xpo.places, xpo.counts[3:4], xf, out=xhr)
        torch.cuda.synchronize()
        xprof = rhx.profile_read()
        rhx.profile_enable(False)
        xboxes = RH.boxes_np(xpo.boxes, xc[0])
        xpb, xub = mem_bytes(xc[1], xboxes, xc[3], F * X)
        result["memory_steps"][f"x{X}"] = {
            "frames": F * X, "n_bins": xc[1],
            "select": mem_row(sel_bytes(F * X, xc[3]), xprof["select"][0] / reps),
            "plan_us": xprof["plan"][0] / reps * 1e3,
            "pack_gather": mem_row(xpb, xprof["gather"][0] / reps),
            "unpack": mem_row(xub, xprof["unpack"][0] / reps)}
        rhx.close()
        del rhx, xf, xi, xhr, xnet, xpo

    if not args.no_temporal:
        # Temporal importance reuse (Sec. 3.2.2) on one chunk of every stream: which frames get a
        # predicted importance map.  It runs before the path and is reported beside it.
        ns, fps = args.temporal_streams, args.temporal_frames
        tF, tau, min_area = ns * fps, 12, 2
        budget = max(ns, tF // 5)
        res = wl.make_residuals(cfg.width, cfg.height, ns, fps, seed=cfg.index)
        rht = RH(frame_w=cfg.width, frame_h=cfg.height, max_frames=tF, halo=cfg.halo, bin_size=cfg.bin_size,
                 max_bins=4, net=cfg.net, weights=blob, precision=cfg.precision)
        d_res = torch.from_numpy(res).cuda()
        t_imp = torch.zeros((tF, rht.mbh, rht.mbw), dtype=torch.float32, device="cuda")
        off = [fps * i for i in range(ns + 1)]
        d_phi = torch.empty(tF, dtype=torch.int64, device="cuda")
        reps, t_us = 10, {}
        for it in range(2):                                           # first round untimed
            rht.profile_enable(it == 1)
            for _ in range(reps):
                rht.temporal_phi(d_res, tau, min_area, out=d_phi)
            if it: t_us["phi"] = rht.profile_read()["temporal"][0] / reps * 1e3
            for _ in range(reps):
                t_alloc, t_sel, t_reuse, t_n = rht.temporal_select(d_phi, off, budget)
            if it: t_us["select"] = rht.profile_read()["temporal"][0] / reps * 1e3
            for _ in range(reps):
                rht.temporal_spread(t_imp, t_sel, t_reuse)
            if it: t_us["spread"] = rht.profile_read()["temporal"][0] / reps * 1e3
        n_pred = int(t_n.cpu()[0])
        phi_bytes = tF * cfg.height * cfg.width * 2 + tF * 8          # residuals read once, Phi written
        spread_bytes = (tF - n_pred) * rht.mbh * rht.mbw * 4 * 2
        result["temporal_reuse"] = {
            "workload": f"{ns} streams x {fps} frames of {cfg.width}x{cfg.height} luma residuals, tau={tau}, min_area={min_area}, budget={budget}",
            "frames": tF, "frames_predicted": n_pred, "us": t_us,
            "phi": {"bound": "hbm", "bytes": phi_bytes, "GB/s": phi_bytes / (t_us["phi"] * 1e-6) / 1e9, "peak": 8000.0,
                    "frac": phi_bytes / (t_us["phi"] * 1e-6) / 1e9 / 8000.0},
            "spread_GB/s": spread_bytes / max(t_us["spread"] * 1e-6, 1e-12) / 1e9}
        if not args.no_cpu_baseline:
            from oracle import temporal as OT
            sub = res[: min(tF, 60)]
            t0 = time.perf_counter()
            o_phi, _ = OT.phi(sub, tau, min_area)
            t1 = time.perf_counter()
            assert np.array_equal(d_phi.cpu().numpy().view(np.uint64)[: len(sub)], o_phi), "temporal leg: Phi differs from the oracle"
            result["temporal_reuse"]["cpu_oracle"] = {"phi_us_per_frame": (t1 - t0) / len(sub) * 1e6, "cores": 1,
                                                      "sample": f"{len(sub)} frames"}
        rht.close()
        del rht, d_res

    fb_ms = None
    if not args.no_frame_based:
        fb_ms = run.frame_based(max(2, args.steps // 4))
        result["frame_based"] = {"ms_per_step": fb_ms, "macroblocks_per_s": F * cfg.mbw * cfg.mbh / (fb_ms * 1e-3),
                                 "region_speedup": fb_ms / ms_step,
                                 "pixel_ratio": F * cfg.width * cfg.height / max(px_lr, 1)}
    other_ms = sum(prof[k][0] for k in ("select", "plan", "gather", "unpack"))
    run.close()
    del run, rh, po

    if not args.box_masked and not args.no_box_masked_leg and not args.exact_border and cfg.precision == "bf16" and cfg.net.channels == 64:
        # The same batch with rh_enhance_masked: the body convs compute only the 8 x 32 cells that a box
        # touches (the other cells hold zeros).  Not the headline: its output differs from rh_enhance's
        # within the receptive field of the skipped cells.
        args.box_masked = True
        rm = Runner(cfg, args, max_box_mbs=args.max_box_mbs, per_layer_tail=args.per_layer_tail)
        args.box_masked = False
        ms_m, prof_m, counts_m = rm.timed(max(3, args.steps // 2), 2)
        sm_m = rm.summary(ms_m, prof_m, counts_m)
        result["box_masked"] = {"ms_per_step": ms_m, "macroblocks_per_s": sm_m["macroblocks_per_s"],
                                "speedup_over_plain": ms_step / ms_m, "live_cell_fraction": rm.live_frac,
                                "kernel_ms_per_step": sm_m["kernel_ms_per_step"],
                                "conv_class_frac": sm_m["conv_class"]["frac_of_peak"]}
        rm.close()
        del rm

    if (not args.needed_region and not args.box_masked and not args.no_needed_region_leg and not args.exact_border
            and not args.per_layer_tail and cfg.precision == "bf16" and cfg.net.channels == 64):
        # The same batch with rh_enhance_needed: every layer computes only the cells within its own radius of a
        # pasted macroblock.  frames_hr and the enhanced pixels are bit-identical to the headline run's; the
        # enhance output outside the pasted macroblocks (which nothing reads) is not produced.
        args.needed_region = True
        rn = Runner(cfg, args, max_box_mbs=args.max_box_mbs)
        args.needed_region = False
        ms_n, prof_n, counts_n = rn.timed(max(3, args.steps // 2), 2)
        sm_n = rn.summary(ms_n, prof_n, counts_n)
        result["needed_region"] = {"ms_per_step": ms_n, "macroblocks_per_s": sm_n["macroblocks_per_s"],
                                   "speedup_over_plain": ms_step / ms_n, "mean_cell_fraction_body_convs": rn.live_frac,
                                   "cell_fraction_tail": rn.tail_frac,
                                   "kernel_ms_per_step": sm_n["kernel_ms_per_step"],
                                   "conv_class_frac": sm_n["conv_class"]["frac_of_peak"],
                                   "output": "frames_hr and enhanced pixels bit-identical to the headline run"}
        rn.close()
        del rn

    if not args.no_other_configs:
        # The other benchmark configurations, GPU legs only (fewer steps): 1, 2 and 5 as listed, and
        # configuration 4 = configuration 3's batch with 5 ... 100 % of the macroblocks selected, for
        # clustered and for iid-uniform importance; region-based time against the frame-based run.
        oc = {}
        o_steps = max(3, args.steps // 4)

        def leg(c, fb=None):
            r = Runner(c, args)
            ms, pr, cn = r.timed(o_steps, 2)
            d = r.summary(ms, pr, cn)
            d["conv_class_frac"] = d.pop("conv_class")["frac_of_peak"]
            d["plan_ms"] = d["kernel_ms_per_step"]["plan"]
            del d["kernel_ms_per_step"]
            if fb is None:
                fb = r.frame_based(2)
            d["frame_based_ms"] = fb
            d["region_speedup"] = fb / ms
            r.close()
            if c.precision == "bf16" and c.net.channels == 64 and not args.per_layer_tail and not args.exact_border and not args.box_masked:
                # the same leg with rh_enhance_needed (pasted pixels bit-identical)
                was, args.needed_region = args.needed_region, True
                rn_ = Runner(c, args)
                args.needed_region = was
                ms_n_, _, _ = rn_.timed(o_steps, 2)
                d["needed_region_ms"] = ms_n_
                d["needed_region_speedup_over_frame_based"] = fb / ms_n_
                rn_.close()
            return d, fb
        for ci in (1, 2, 5):
            c = wl.config(ci)
            oc[c.name], _ = leg(c)
        plain3 = (args.config in (3, 4) and not args.exact_border and not args.per_layer_tail and args.bin_size is None
                  and not args.max_box_mbs)
        sweep, fb4 = {}, (fb_ms if plain3 else None)
        for kind in ("clustered", "uniform"):
            for frac in (0.05, 0.10, 0.20, 0.50, 1.00):
                d, fb4 = leg(wl.replace(wl.config(4), frac=frac, importance=kind), fb4)
                sweep[f"{kind}_{int(frac * 100)}pct"] = d
        oc["cfg4_fraction_sweep"] = sweep
        result["other_configs"] = oc

    if not args.no_planner and cfg.precision == "bf16":
        # Planner-lite (Sec. 3.4): bin size and bins per launch from the cost curve kept in the tree and
        # the packer's bin counts for this batch; the chosen geometry is then timed end to end.
        from paper_2407_16990_amd import planner as PL
        if os.path.exists(PL.CURVE_FILE):
            curve = PL.load_curve()
            cands = PL.measure_candidates(d_frames, d_imp, seg_rows, cfg.net, blob, cfg.precision, cfg.halo,
                                          [(Sx, 0) for Sx in sorted(curve)])
            ch = PL.choose(curve, cands, other_ms=other_ms)
            pl = {"candidates": [{"bin_size": c.bin_size, "n_bins": c.n_bins} for c in cands],
                  "chosen": {"bin_size": ch.bin_size, "bins_per_launch": ch.bins_per_launch, "launches": ch.launches,
                             "predicted_ms_per_step": ch.ms_per_batch, "predicted_macroblocks_per_s": ch.macroblocks_per_s}}
            if ch.bin_size != S:
                r2 = Runner(wl.replace(cfg, bin_size=ch.bin_size), args)
                ms2, _, cn2 = r2.timed(max(3, args.steps // 2), 2)
                pl["chosen"].update({"measured_ms_per_step": ms2, "measured_macroblocks_per_s": cn2[3] / (ms2 * 1e-3),
                                     "speedup_over_configured_bin_size": ms_step / ms2})
                r2.close()
                if cfg.net.channels == 64 and not args.per_layer_tail and not args.exact_border and not args.box_masked:
                    # the chosen geometry with rh_enhance_needed (same pasted pixels): the two gains compose
                    was, args.needed_region = args.needed_region, True
                    r3 = Runner(wl.replace(cfg, bin_size=ch.bin_size), args)
                    args.needed_region = was
                    ms3, _, cn3 = r3.timed(max(3, args.steps // 2), 2)
                    pl["chosen"].update({"needed_region_ms_per_step": ms3, "needed_region_macroblocks_per_s": cn3[3] / (ms3 * 1e-3)})
                    r3.close()
            else:
                pl["chosen"].update({"measured_ms_per_step": ms_step, "speedup_over_configured_bin_size": 1.0})
            result["planner_lite"] = pl

    if not args.no_cpu_baseline:
        import oracle
        cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        t = time.perf_counter()
        o_mask, o_list = oracle.select(imp, segs)
        pl = oracle.plan(o_mask, imp, cfg.halo, S)
        o_bins = oracle.gather(frames, pl.boxes, cfg.halo, S, pl.n_bins)
        t_meta = time.perf_counter() - t
        nb_s = min(pl.n_bins, cores)
        t = time.perf_counter()
        o_net = oracle.sr_forward(cfg.net, blob, o_bins[:nb_s])
        t_sr = time.perf_counter() - t
        # paste on one frame's worth of the batch, scaled to all frames
        t = time.perf_counter()
        oracle.unpack(frames[:1], s, o_net, pl.places[:0])
        t_un = (time.perf_counter() - t) * F
        est = t_meta + t_sr * pl.n_bins / nb_s + t_un
        result["cpu_baseline"] = {"value": len(o_list) / est, "unit": "MB/s", "cores": cores, "kind": "oracle",
                                  "sample": f"select+plan+gather in full ({t_meta:.3f} s); SR on {nb_s} of {pl.n_bins} bins "
                                            f"({t_sr:.1f} s, one bin per core), scaled by bin count; bilinear base on 1 of {F} "
                                            f"frames scaled ({t_un:.2f} s)"}
    print(json.dumps(result))


if __name__ == "__main__":
    main()
