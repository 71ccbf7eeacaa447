"""Planner-lite on the GPU (Sec. 3.4): the geometry it chooses for the benchmark batch from the
tracked cost curve and the packer's own bin counts must not be slower than the configured one."""
import time

import pytest
import torch

import workloads as wl
from paper_2407_16990_amd import RH, planner as PL

pytestmark = pytest.mark.gpu


def _ms_per_step(cfg, frames, imp, seg_rows, blob, steps=8):
    s, S, F = cfg.net.scale, cfg.bin_size, cfg.n_frames
    rh = RH(frame_w=cfg.width, frame_h=cfg.height, max_frames=F, halo=cfg.halo, bin_size=S, max_bins=256, net=cfg.net,
            weights=blob, precision=cfg.precision)
    mask, lst, n_sel = rh.select_regions(imp, seg_rows)
    po = rh.pack(frames, imp, mask, lst, n_sel)
    nb = rh.read_counts(po.counts)[1]
    net_out = torch.empty((nb, S * s, S * s, 3), dtype=torch.float32, device="cuda")
    hr = torch.empty((F, cfg.height * s, cfg.width * s, 3), dtype=torch.uint8, device="cuda")

    def step():
        m, l, n = rh.select_regions(imp, seg_rows)
        rh.pack(frames, imp, m, l, n, out=po)
        rh.enhance(po.bins, n=nb, n_valid=po.counts[1:2], out=net_out)
        rh.unpack(net_out, po.places, po.counts[3:4], frames, out=hr)
    for _ in range(3):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / steps * 1e3
    rh.close()
    return ms


def test_planner_choice_is_not_slower_than_the_configured_bin_size():
    cfg = wl.config(3)
    frames = torch.from_numpy(wl.make_frames(cfg)).cuda()
    imp = torch.from_numpy(wl.make_importance(cfg)).cuda()
    seg_rows = [tuple(r) for r in wl.make_segments(cfg).tolist()]
    blob = wl.make_weights(cfg.net, cfg.weight_seed, cfg.precision)
    curve = PL.load_curve()
    cands = PL.measure_candidates(frames, imp, seg_rows, cfg.net, blob, cfg.precision, cfg.halo, [(S, 0) for S in sorted(curve)])
    assert {c.bin_size for c in cands} == set(curve) and all(c.n_selected == 1632 for c in cands)
    ch = PL.choose(curve, cands)
    base = _ms_per_step(cfg, frames, imp, seg_rows, blob)
    chosen = _ms_per_step(wl.replace(cfg, bin_size=ch.bin_size), frames, imp, seg_rows, blob) if ch.bin_size != cfg.bin_size else base
    print(f"planner-lite: S={ch.bin_size}, {ch.bins_per_launch} bins per launch, predicted enhance {ch.ms_per_batch:.2f} ms; "
          f"measured step {chosen:.2f} ms against {base:.2f} ms at S={cfg.bin_size}", flush=True)
    assert chosen <= base * 1.03
    # a launch budget below the whole batch's cost splits the batch, and every launch fits the budget
    tight = PL.choose(curve, cands, budget_ms=2.0)
    assert tight.launches >= 2 and PL.cost(curve[tight.bin_size], tight.bins_per_launch) <= 2.0
