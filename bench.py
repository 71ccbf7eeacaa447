#!/usr/bin/env python3
"""Benchmark of the region-aware enhancer hot path on one MI355X.

A step = one pass of the whole path (rh_select_regions -> rh_pack -> rh_enhance -> rh_unpack)
over one batch of synthetic input already resident in HBM.  Workload: configuration 3 of the
benchmark list (16 frames 480x272, EDSR-baseline x4, top 20 % macroblocks, halo 10, 128x128
bins, bf16), the one the headline metric "enhanced macroblocks/s" is quoted on.

Prints ONE JSON line with the metric, the roofline of the dominant kernel (the bf16 MFMA conv,
timed with HIP events inside the timed region), the CPU oracle timed on a bounded sample
(cpu_baseline), and the 100 %-macroblock frame-based run on the GPU for comparison.
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

MFMA_BF16_PEAK = 2.5e15   # dense bf16 MFMA, FLOP/s (MI355X published)
FP32_VALU_PEAK = 157.3e12  # fp32 vector ALUs, FLOP/s (MI355X published)
# HBM bytes per launch of the dominant kernel class on the default workload, from the rocprofv3
# FETCH_SIZE / WRITE_SIZE runs summarised in profiles/conv_mfma_cfg3_hbm_counters.md (scaled by
# the plain-copy calibration); not measured live, so only reported for that workload.
MEASURED_TRAFFIC = {"cfg3_16x480x272_edsr64_x4_bf16": 499.0e6}
CONV_KERNEL = {64: "k_conv_mfma_duo<SKIP,RELU,10> (bf16-output 64-channel convs: ReLU, skip-add and plain instantiations)",
               32: "k_conv_mfma<32,1,16,false,SKIP,RELU> (bf16-output 32-channel convs)"}


def conv_flops_per_lr_pixel(net):
    """Algorithmic FLOPs of the C-input/bf16-output convs (the profiled kernel class) per
    packed low-resolution pixel: 18*cin*cout per output pixel at the layer's resolution."""
    C, s = net.channels, net.scale
    body = 2 * net.n_blocks + (1 if net.topology == "edsr" else 0)
    fl = body * 18 * C * C
    launches = body
    if net.topology == "edsr":
        if s == 4:
            fl += 18 * C * 4 * C + 4 * 18 * C * 4 * C
            launches += 2
        else:
            fl += 18 * C * C * s * s
            launches += 1
    return fl, launches


def total_flops_per_lr_pixel(net):
    C, s = net.channels, net.scale
    fl, _ = conv_flops_per_lr_pixel(net)
    fl += 18 * 3 * C
    fl += (s * s * 18 * C * 3) if net.topology == "edsr" else 18 * C * 3 * s * s
    return fl


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-frame-based", action="store_true")
    ap.add_argument("--fraction", type=float, default=None,
                    help="override the selected fraction of the configuration (the fraction sweep of configuration 4)")
    ap.add_argument("--importance", choices=["clustered", "uniform"], default=None,
                    help="override the importance recipe (uniform = iid, isolated macroblocks: the packer's worst case)")
    ap.add_argument("--exact-border", action="store_true",
                    help="enhance with rh_enhance_exact (per-layer zeroing of the out-of-frame part of the boxes)")
    ap.add_argument("--bin-size", type=int, default=None, help="override the bin side S (pixels)")
    ap.add_argument("--max-box-mbs", type=int, default=0,
                    help="Partition's preset size in macroblocks (0 = the largest that fits a bin; 1 = every "
                         "macroblock its own box, the paper's MB-packing / Block policy)")
    ap.add_argument("--policy-study", type=int, default=0, metavar="N",
                    help="occupy ratio (selected-MB pixels / packed pixels) of the packing policies over N random "
                         "importance maps of the configuration: importance-density order (the paper's), the same "
                         "with RotatePacking, large-item-first order, and one box per macroblock (MB packing)")
    ap.add_argument("--mem-batch", type=int, default=16, metavar="X",
                    help="also time the memory-bound steps (pack gather, unpack) on X copies of the batch, where "
                         "they are large enough to be bandwidth- rather than launch-bound (0 = skip)")
    ap.add_argument("--no-temporal", action="store_true",
                    help="skip the temporal importance reuse leg (Sec. 3.2.2; reported beside the path, not in `value`)")
    ap.add_argument("--temporal-streams", type=int, default=10, help="streams of the temporal leg's chunk")
    ap.add_argument("--temporal-frames", type=int, default=30, help="frames per stream of the temporal leg's chunk")
    ap.add_argument("--sync-counts", action="store_true",
                    help="read the bin count back to the host after rh_pack (one synchronisation per step) and "
                         "enhance exactly that many bins, instead of passing the device-side count")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MiB",
                    help="also run one plain device copy of this many MiB (reference for scaling rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE counters)")
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
    F, s = cfg.n_frames, cfg.net.scale
    frames, imp, segs = wl.make_frames(cfg), wl.make_importance(cfg), wl.make_segments(cfg)
    blob = wl.make_weights(cfg.net, cfg.weight_seed, cfg.precision)
    # room for the packer's worst case (isolated macroblocks: one box each)
    max_bins = 512 if (cfg.index == 5 or cfg.importance == "uniform" or args.max_box_mbs == 1) else 256
    max_bins = max_bins * max(1, (128 // cfg.bin_size) ** 2)
    rh = RH(frame_w=cfg.width, frame_h=cfg.height, max_frames=F, halo=cfg.halo, bin_size=cfg.bin_size,
            max_bins=max_bins, net=cfg.net, weights=blob, precision=cfg.precision, max_box_mbs=args.max_box_mbs)
    d_frames = torch.from_numpy(frames).cuda()
    d_imp = torch.from_numpy(imp).cuda()
    seg_rows = [tuple(r) for r in segs.tolist()]
    S = cfg.bin_size
    # all outputs are allocated once, outside the timed region
    po = None
    net_out = torch.empty((max_bins, S * s, S * s, 3), dtype=torch.float32, device="cuda")
    hr = torch.empty((F, cfg.height * s, cfg.width * s, 3), dtype=torch.uint8, device="cuda")

    def step():
        nonlocal po
        mask, lst, n_sel = rh.select_regions(d_imp, seg_rows)
        po = rh.pack(d_frames, d_imp, mask, lst, n_sel, out=po)
        if args.exact_border:
            rh.enhance_exact(po.bins, po.boxes, po.counts, n=max_bins, n_valid=po.counts[1:2], out=net_out)
        elif args.sync_counts:
            rh.enhance(po.bins, n=rh.read_counts(po.counts)[1], out=net_out)
        else:
            rh.enhance(po.bins, n=max_bins, n_valid=po.counts[1:2], out=net_out)   # device-side bin count
        rh.unpack(net_out, po.places, po.counts[3:4], d_frames, out=hr)

    if args.calibrate_copy:
        src = torch.full((args.calibrate_copy << 20,), 7, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    counts = rh.read_counts(po.counts)
    n_boxes, n_bins, _, k_sel = counts
    rh.profile_enable(True)
    rh.profile_read()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    prof = rh.profile_read()
    rh.profile_enable(False)

    ms_step = dt / args.steps * 1e3
    mbs_per_s = k_sel * args.steps / dt
    out_mpix = F * cfg.height * s * cfg.width * s * args.steps / dt / 1e6
    px_lr = n_bins * S * S
    conv_fl, conv_launches = conv_flops_per_lr_pixel(cfg.net)
    if cfg.precision != "bf16":
        # the fp32 path times all its layers as one class: direct convs on the vector ALUs
        conv_fl, conv_launches = total_flops_per_lr_pixel(cfg.net), len(wl.net_layers(cfg.net))
    conv_ms, conv_n = prof["conv"]
    avg_launch_s = conv_ms / max(conv_n, 1) * 1e-3
    flop_per_launch = conv_fl * px_lr / conv_launches
    achieved = flop_per_launch / avg_launch_s if avg_launch_s > 0 else 0.0
    PEAK = MFMA_BF16_PEAK if cfg.precision == "bf16" else FP32_VALU_PEAK

    result = {
        "metric": "enhanced macroblocks/s",
        "value": mbs_per_s, "unit": "MB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.precision == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": cfg.name, "frames": F, "frame": [cfg.width, cfg.height], "scale": s,
                   "selected_fraction": cfg.frac, "halo": cfg.halo, "bin_size": S,
                   "n_selected": k_sel, "n_boxes": n_boxes, "n_bins": n_bins,
                   "occupy_ratio": 256.0 * k_sel / (n_bins * S * S) if n_bins else 0.0},
        "output_mpixel_per_s": out_mpix,
        "kernel_ms_per_step": {k: v[0] / args.steps for k, v in prof.items()},
        "roofline": {"bound": "mfma" if cfg.precision == "bf16" else "alu",
                     "kernel": CONV_KERNEL.get(cfg.net.channels, "k_conv_mfma") if cfg.precision == "bf16" else "k_conv3x3_f32 (all layers)",
                     "achieved": achieved / 1e12,
                     "peak": PEAK / 1e12, "unit": "TFLOP/s", "frac": achieved / PEAK,
                     "traffic": MEASURED_TRAFFIC.get(cfg.name), "avg_launch_us": avg_launch_s * 1e6, "launches_per_step": conv_n / args.steps,
                     "flop_per_launch": flop_per_launch},
        "enhance_tflops_all_layers": total_flops_per_lr_pixel(cfg.net) * px_lr /
                                     max(sum(prof[k][0] for k in ("head", "conv", "conv_last")) / args.steps * 1e-3, 1e-12) / 1e12,
    }

    # ---- the memory-bound steps: algorithmic bytes / event time, at batch size and at X batches ----
    def mem_bytes(nb, boxes_host, nsel, nf):
        box_px = sum((16 * int(b["wmb"]) + 2 * cfg.halo) * (16 * int(b["hmb"]) + 2 * cfg.halo) for b in boxes_host)
        pack_b = nb * S * S * 3 + box_px * 3                      # every bin byte written, box pixels read
        unpack_b = nf * cfg.height * s * cfg.width * s * 3 + nf * cfg.height * cfg.width * 3 + nsel * (16 * s) ** 2 * 3 * 4
        return pack_b, unpack_b

    boxes_host = RH.boxes_np(po.boxes, n_boxes)
    pb, ub = mem_bytes(n_bins, boxes_host, k_sel, F)
    sel_bytes = lambda nf, nsel: nf * rh.mbh * rh.mbw * 5 + nsel * 4          # 4 B read + 1 B mask per MB, 4 B per selected MB
    sb = sel_bytes(F, k_sel)
    result["memory_steps"] = {
        "select": {"bytes": sb, "us": prof["select"][0] / args.steps * 1e3, "GB/s": sb / (prof["select"][0] / args.steps * 1e-3) / 1e9,
                   "note": "latency-bound: tens of kilobytes"},
        "pack_gather": {"bytes": pb, "us": prof["gather"][0] / args.steps * 1e3, "GB/s": pb / (prof["gather"][0] / args.steps * 1e-3) / 1e9},
        "unpack": {"bytes": ub, "us": prof["unpack"][0] / args.steps * 1e3, "GB/s": ub / (prof["unpack"][0] / args.steps * 1e-3) / 1e9},
        "hbm_peak_GB/s": 8000.0}
    if args.mem_batch > 0:
        X = args.mem_batch
        rhx = RH(frame_w=cfg.width, frame_h=cfg.height, max_frames=F * X, halo=cfg.halo, bin_size=cfg.bin_size,
                 max_bins=max_bins * X, net=cfg.net, weights=blob, precision=cfg.precision,
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
            "select": {"bytes": sel_bytes(F * X, xc[3]), "us": xprof["select"][0] / reps * 1e3,
                       "GB/s": sel_bytes(F * X, xc[3]) / (xprof["select"][0] / reps * 1e-3) / 1e9},
            "pack_gather": {"bytes": xpb, "us": xprof["gather"][0] / reps * 1e3, "GB/s": xpb / (xprof["gather"][0] / reps * 1e-3) / 1e9},
            "unpack": {"bytes": xub, "us": xprof["unpack"][0] / reps * 1e3, "GB/s": xub / (xprof["unpack"][0] / reps * 1e-3) / 1e9}}
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
        del rht, d_res

    if args.policy_study > 0:
        pols = {"density": dict(), "density+rotate": dict(rotate=True), "area": dict(sort_policy="area"),
                "area+rotate": dict(sort_policy="area", rotate=True), "mb_packing": dict(max_box_mbs=1)}
        ctxs = {k: RH(frame_w=cfg.width, frame_h=cfg.height, max_frames=F, halo=cfg.halo, bin_size=cfg.bin_size,
                      max_bins=4 * max_bins, net=cfg.net, weights=blob, precision=cfg.precision, **kw)
                for k, kw in pols.items()}
        occ = {k: [] for k in pols}
        plan_ms = {k: 0.0 for k in pols}
        for it in range(args.policy_study):
            ci = wl.replace(cfg, index=1000 + it)                     # another seed of the same recipe
            x_imp = torch.from_numpy(wl.make_importance(ci)).cuda()
            x_segs = [tuple(r) for r in wl.make_segments(ci).tolist()]
            for k, c in ctxs.items():
                c.profile_enable(True)
                m_, l_, n_ = c.select_regions(x_imp, x_segs)
                o_ = c.pack(d_frames, x_imp, m_, l_, n_)
                cnt = c.read_counts(o_.counts)
                plan_ms[k] += c.profile_read()["plan"][0]
                occ[k].append(256.0 * cnt[3] / (cnt[1] * S * S) if cnt[1] else 0.0)
        result["policy_study"] = {"n": args.policy_study, "bin_size": S, "halo": cfg.halo}
        for k, v in occ.items():
            a = np.asarray(v)
            result["policy_study"][k] = {"occupy_mean": float(a.mean()), "occupy_p05": float(np.percentile(a, 5)),
                                         "occupy_p10": float(np.percentile(a, 10)), "occupy_p50": float(np.percentile(a, 50)),
                                         "plan_ms_mean": plan_ms[k] / args.policy_study}
        for c in ctxs.values():
            c.close()

    if not args.no_frame_based:
        # 100 % of the macroblocks: rh_enhance on whole frames + identity placement
        places, n_pl = rh.identity_places(F)
        fb_net = torch.empty((F, cfg.height * s, cfg.width * s, 3), dtype=torch.float32, device="cuda")

        def fb_step():
            rh.enhance(d_frames, out=fb_net)
            rh.unpack(fb_net, places, n_pl, d_frames, out=hr)
        fb_step()
        torch.cuda.synchronize()
        n_fb = max(2, args.steps // 4)
        t0 = time.perf_counter()
        for _ in range(n_fb):
            fb_step()
        torch.cuda.synchronize()
        fdt = (time.perf_counter() - t0) / n_fb
        result["frame_based"] = {"ms_per_step": fdt * 1e3, "macroblocks_per_s": F * cfg.mbw * cfg.mbh / fdt,
                                 "region_speedup": fdt * 1e3 / ms_step,
                                 "pixel_ratio": F * cfg.width * cfg.height / max(px_lr, 1)}

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
