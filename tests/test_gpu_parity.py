"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.
Bars: bit-exact selection, plan and packed bytes; pixels rel-L2 <= 1e-5 on the fp32 path and
<= 1e-2 with max abs <= 2/255 on the bf16 path."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from paper_2407_16990_amd import RH, RhError
from gpu_common import bf16_max_abs_bar, check_net, check_select_and_plan, dev, gpu_select, make_rh, rel_l2

pytestmark = pytest.mark.gpu


def full_path_check(cfg, n_frames=None, precision=None, segs=None, max_bins=None, sort_policy="density", rotate=False,
                    expect_turned=False, per_layer_tail=False, masked=False, needed=False):
    F = cfg.n_frames if n_frames is None else n_frames
    precision = precision or cfg.precision
    frames, imp = wl.make_frames(cfg, F), wl.make_importance(cfg, F)
    segs = wl.make_segments(cfg, F) if segs is None else segs
    blob = wl.make_weights(cfg.net, cfg.weight_seed, precision)
    rh = make_rh(cfg, blob, F, precision=precision, max_bins=max_bins, sort_policy=sort_policy, rotate=rotate,
                 per_layer_tail=per_layer_tail)
    o_plan, po, (d_frames, d_imp, o_bins) = check_select_and_plan(rh, cfg, frames, imp, segs, sort_policy=sort_policy,
                                                                  rotate=rotate)
    if expect_turned:
        assert o_plan.boxes[:, 5].sum() > 0, "the case is meant to turn at least one box"
    s = cfg.net.scale
    # enhance: both the exact-N call and the device-count call
    if needed:      # needed-region mode: defined on the pasted macroblocks only, and there it is the plain mode's output
        on = np.zeros((o_plan.n_bins, cfg.bin_size * s, cfg.bin_size * s), dtype=bool)
        for g, box, b, px, py in o_plan.places.tolist():
            on[b, py * s:(py + 16) * s, px * s:(px + 16) * s] = True
        g_plain = rh.enhance(po.bins, n=o_plan.n_bins)
        g_net = torch.full_like(g_plain, float("nan"))           # whatever the mode leaves unwritten stays NaN
        rh.enhance_needed(po.bins, po.places, po.counts, n=o_plan.n_bins, out=g_net)
        assert torch.equal(g_net[torch.from_numpy(on).cuda()], g_plain[torch.from_numpy(on).cuda()]), "not bit-identical on the pasted pixels"
        o_net = oracle.sr_forward(cfg.net, blob, o_bins)
        check_net(g_net.cpu().numpy()[on], o_net[on], precision, f"{cfg.name} n_bins={o_plan.n_bins} needed-region, pasted pixels")
        g_net2 = torch.full_like(g_plain, float("nan"))
        rh.enhance_needed(po.bins, po.places, po.counts, n=o_plan.n_bins, n_valid=po.counts[1:2], out=g_net2)
        assert torch.equal(g_net2[torch.from_numpy(on).cuda()], g_plain[torch.from_numpy(on).cuda()])
        del g_net2, g_plain
    elif masked:    # box-masked mode: the body skips the cells no box touches, which hold zeros
        keep = oracle.cell_keep(o_plan.boxes, cfg.halo, cfg.bin_size, o_plan.n_bins)
        print(f"[{cfg.name}] live cell fraction {keep.mean():.3f}", flush=True)
        assert keep.mean() < 1.0, "the case is meant to have cells that no box touches"
        g_net = rh.enhance_masked(po.bins, po.boxes, po.counts, n=o_plan.n_bins)
        o_net = oracle.sr_forward(cfg.net, blob, o_bins, keep, body_only=True)
    else:
        g_net = rh.enhance(po.bins, n=o_plan.n_bins)
        o_net = oracle.sr_forward(cfg.net, blob, o_bins)
    tol = 1e-5 if precision == "fp32" else 1e-2
    if not needed:
        check_net(g_net.cpu().numpy(), o_net, precision, f"{cfg.name} n_bins={o_plan.n_bins}{' masked' if masked else ''}")
    g_net2 = None if needed else torch.zeros_like(g_net)
    if needed:
        pass
    elif masked:
        rh.enhance(po.bins, n=o_plan.n_bins, out=g_net2)           # a plain call in between leaves other values in the workspace
        assert not torch.equal(g_net, g_net2), "the masked mode is a different function"
        rh.enhance_masked(po.bins, po.boxes, po.counts, n=o_plan.n_bins, n_valid=po.counts[1:2], out=g_net2)
    else:
        rh.enhance(po.bins, n=o_plan.n_bins, n_valid=po.counts[1:2], out=g_net2)
    assert needed or torch.equal(g_net, g_net2)
    # unpack
    hr, sel = rh.unpack(g_net, po.places, po.counts[3:4], d_frames, want_sel=True)
    o_hr, o_sel = oracle.unpack(frames, s, o_net, o_plan.places, place_rot=o_plan.place_rot)
    k = len(o_plan.places)
    g_sel = sel[:k].cpu().numpy()
    e_sel = rel_l2(g_sel, o_sel)
    print(f"[{cfg.name}/{precision}] enhanced pixels rel-L2={e_sel:.3e} max abs={np.abs(g_sel - o_sel).max():.3e}", flush=True)
    assert e_sel <= tol
    g_hr = hr.cpu().numpy()
    B = 16 * s
    selmask = np.kron(oracle.select(imp, segs)[0], np.ones((B, B), dtype=np.uint8)).astype(bool)
    assert np.array_equal(g_hr[~selmask], o_hr[~selmask]), "unselected macroblocks must be the bilinear base exactly"
    d = np.abs(g_hr.astype(np.int16) - o_hr.astype(np.int16))[selmask]
    if precision == "fp32":
        assert d.max() <= 1 and (d > 0).mean() < 1e-3
    else:
        bar = bf16_max_abs_bar(o_net)
        assert np.abs(g_sel - o_sel).max() <= bar and d.max() <= round(bar * 255)
    rh.close()


def test_cfg1_whole_path_fp32():
    full_path_check(wl.config(1))


@pytest.mark.parametrize("net", [wl.Net("res", 8, 2, 2, 0.05), wl.Net("edsr", 8, 2, 2, 0.05),
                                 wl.Net("edsr", 8, 1, 3, 0.05), wl.Net("edsr", 12, 2, 4, 0.05)])
def test_small_topologies_fp32(net):
    cfg = wl.replace(wl.config(1), net=net, n_frames=2, halo=5, frac=0.3)
    full_path_check(cfg)


@pytest.mark.parametrize("ci", [1, 2, 3, 5])
def test_metadata_and_bytes_at_full_size(ci):
    cfg = wl.config(ci)
    frames, imp = wl.make_frames(cfg), wl.make_importance(cfg)
    blob = wl.make_weights(wl.Net("plain", 4, 2, cfg.net.scale), 0, "fp32")
    rh = make_rh(wl.replace(cfg, net=wl.Net("plain", 4, 2, cfg.net.scale)), blob, precision="fp32")
    check_select_and_plan(rh, cfg, frames, imp, wl.make_segments(cfg))
    rh.close()


def test_contexts_of_different_sizes_coexist():
    """A small context created after a large one must not shrink what the large one may launch:
    the planning kernels' shared-memory limit belongs to the kernel, not to a context."""
    big, small = wl.config(5), wl.config(1)
    net = wl.Net("plain", 4, 2, 2)
    blob = wl.make_weights(net, 0, "fp32")
    rh_big = make_rh(wl.replace(big, net=wl.Net("plain", 4, 2, big.net.scale)),
                     wl.make_weights(wl.Net("plain", 4, 2, big.net.scale), 0, "fp32"), precision="fp32")
    rh_small = make_rh(wl.replace(small, net=net), blob, precision="fp32")
    check_select_and_plan(rh_small, small, wl.make_frames(small), wl.make_importance(small), wl.make_segments(small))
    check_select_and_plan(rh_big, big, wl.make_frames(big), wl.make_importance(big), wl.make_segments(big))
    check_select_and_plan(rh_small, small, wl.make_frames(small), wl.make_importance(small), wl.make_segments(small))
    rh_big.close()
    rh_small.close()


@pytest.mark.parametrize("frac,kind", [(0.05, "clustered"), (0.5, "clustered"), (1.0, "clustered"),
                                       (0.1, "uniform"), (0.2, "uniform"), (0.5, "uniform")])
def test_sweep_metadata(frac, kind):
    cfg = wl.replace(wl.config(4), frac=frac, importance=kind)
    frames, imp = wl.make_frames(cfg), wl.make_importance(cfg)
    net = wl.Net("plain", 4, 2, 4)
    rh = make_rh(wl.replace(cfg, net=net), wl.make_weights(net, 0, "fp32"), precision="fp32")
    check_select_and_plan(rh, cfg, frames, imp, wl.make_segments(cfg))
    rh.close()


@pytest.mark.parametrize("levels", [10, 2, 1])
def test_tie_stress_and_connectivity(levels):
    cfg = wl.replace(wl.config(2), quantize_levels=levels, n_frames=4)
    frames, imp = wl.make_frames(cfg), wl.make_importance(cfg)
    net = wl.Net("plain", 4, 2, 2)
    for conn, T in [(8, 0), (4, 2), (8, 1), (4, 5)]:
        rh = make_rh(wl.replace(cfg, net=net), wl.make_weights(net, 0, "fp32"), precision="fp32",
                     connectivity=conn, max_box_mbs=T)
        segs = np.array([[0, 1, 300], [1, 3, 911], [3, 4, 0]], dtype=np.uint32)
        check_select_and_plan(rh, cfg, frames, imp, segs, conn=conn, T=T or None)
        rh.close()


@pytest.mark.parametrize("w,h,kind,conn,T,rotate", [(1056, 48, "uniform", 8, 0, False), (1072, 80, "clustered", 4, 2, True),
                                                    (64, 1056, "uniform", 8, 1, False), (1040, 1040, "clustered", 8, 0, False)])
def test_plan_of_frames_wider_than_64_macroblocks(w, h, kind, conn, T, rotate):
    """Frames of more than 64 macroblocks a side are planned by the general multi-launch kernels
    (the one-launch kernel keeps a frame's rows in 64-bit masks, one row per lane)."""
    cfg = wl.replace(wl.config(1), n_frames=2, width=w, height=h, importance=kind, frac=0.3, halo=4, bin_size=96)
    frames, imp = wl.make_frames(cfg), wl.make_importance(cfg)
    net = wl.Net("plain", 4, 2, 2)
    rh = make_rh(wl.replace(cfg, net=net), wl.make_weights(net, 0, "fp32"), precision="fp32", connectivity=conn,
                 max_box_mbs=T, rotate=rotate)
    check_select_and_plan(rh, cfg, frames, imp, wl.make_segments(cfg), conn=conn, T=T or None, rotate=rotate)
    rh.close()


def test_select_specials_threshold_and_edges():
    cfg = wl.replace(wl.config(1), n_frames=3)
    imp = wl.make_importance(cfg)
    imp[0, 0, :5] = [np.nan, -0.0, 0.0, np.inf, -np.inf]
    imp[1, 3, 3] = np.nan
    net = wl.Net("plain", 4, 2, 2)
    rh = make_rh(wl.replace(cfg, net=net), wl.make_weights(net, 0, "fp32"), precision="fp32")
    per = cfg.mbw * cfg.mbh
    for segs in ([[0, 3, 0]], [[0, 3, 1]], [[0, 3, 3 * per]], [[0, 3, 3 * per - 1]], [[0, 3, 10 ** 6]],
                 [[0, 1, 50], [1, 2, 239], [2, 3, 240]], [[1, 2, 17]], []):
        o_mask, o_list = oracle.select(imp, np.array(segs, dtype=np.uint32).reshape(-1, 3))
        g_mask, g_list, _ = gpu_select(rh, imp, segs)
        assert np.array_equal(g_mask, o_mask) and np.array_equal(g_list, o_list), segs
    for thr in (0.5, 0.0, -1.0, 1e9, float("nan"), float("-inf")):
        segs = np.array([[0, 2, 0], [2, 3, 0]], dtype=np.uint32)
        t = np.array([thr, 0.3], dtype=np.float32)
        o_mask, o_list = oracle.select(imp, segs, "threshold", t)
        g_mask, g_list, _ = gpu_select(rh, imp, [(0, 2, 0, thr), (2, 3, 0, 0.3)], "threshold")
        assert np.array_equal(g_mask, o_mask) and np.array_equal(g_list, o_list), thr
    rh.close()


def test_empty_selection_and_overflow_and_errors():
    cfg = wl.replace(wl.config(1), n_frames=2)
    frames, imp = wl.make_frames(cfg), wl.make_importance(cfg)
    net = wl.Net("plain", 4, 2, 2)
    blob = wl.make_weights(net, 0, "fp32")
    c2 = wl.replace(cfg, net=net)
    rh = make_rh(c2, blob, precision="fp32")
    o_plan, po, _ = check_select_and_plan(rh, cfg, frames, imp, np.array([[0, 2, 0]], dtype=np.uint32))
    assert o_plan.n_bins == 0
    hr, _ = rh.unpack(torch.zeros((1, 128, 128, 3), device="cuda"), po.places, po.counts[3:4], dev(frames))
    assert np.array_equal(hr.cpu().numpy()[0], oracle.bilinear(frames[0], 2))
    rh.close()
    # capacity: 3 bins allowed, more needed
    rh = make_rh(c2, blob, precision="fp32", max_bins=3)
    segs = np.array([[0, 2, 200]], dtype=np.uint32)
    o_plan, po, _ = check_select_and_plan(rh, cfg, frames, imp, segs, max_bins=3)
    assert o_plan.overflow
    with pytest.raises(RhError) as ei:
        rh.read_counts(po.counts)
    assert ei.value.status == 3
    # overflowed MBs stay bilinear, placed ones are enhanced: compare with the oracle end to end
    g_net = rh.enhance(po.bins, n=3)
    hr, _ = rh.unpack(g_net, po.places, po.counts[3:4], dev(frames))
    o_net = oracle.sr_forward(net, blob, oracle.gather(frames, o_plan.boxes, cfg.halo, cfg.bin_size, 3))
    o_hr, _ = oracle.unpack(frames, 2, o_net, o_plan.places)
    assert np.abs(hr.cpu().numpy().astype(int) - o_hr.astype(int)).max() <= 1
    # argument errors are reported, not crashed on
    with pytest.raises(RhError):
        rh.select_regions(dev(imp), [(0, 3, 5)])
    with pytest.raises(RhError):
        rh.select_regions(dev(imp), [(1, 2, 5), (0, 1, 5)])
    with pytest.raises(RhError):
        RH(frame_w=12, frame_h=64, max_frames=1, halo=4, bin_size=64, max_bins=4, net=net, weights=blob, precision="fp32")
    with pytest.raises(RhError):
        RH(frame_w=64, frame_h=64, max_frames=1, halo=30, bin_size=64, max_bins=4, net=net, weights=blob, precision="fp32")
    with pytest.raises(RhError):
        RH(frame_w=64, frame_h=64, max_frames=1, halo=4, bin_size=64, max_bins=4, net=net, weights=blob[:-1], precision="fp32")
    rh.close()
    # bf16 path: an image whose activations would pass 2 GiB is refused before anything is launched or allocated
    # (layer by layer the x4 net holds 64 channels at the output resolution)
    net64 = wl.Net("edsr", 64, 1, 4, 0.02)
    rh2 = RH(frame_w=64, frame_h=64, max_frames=1, halo=4, bin_size=64, max_bins=4, net=net64,
             weights=wl.make_weights(net64, 0, "bf16"), precision="bf16", per_layer_tail=True)
    with pytest.raises(RhError) as ei:
        rh2.enhance(torch.zeros((1, 1100, 1100, 3), dtype=torch.uint8, device="cuda"))   # 4400 x 4400 x 128 B > 2 GiB
    assert "2 GiB" in str(ei.value)
    rh2.close()


def test_frame_based_run_fp32_matches_oracle():
    """100 % of the macroblocks through rh_enhance on whole frames + identity placement."""
    cfg = wl.replace(wl.config(1), n_frames=2)
    frames = wl.make_frames(cfg)
    blob = wl.make_weights(cfg.net, 0, "fp32")
    rh = make_rh(cfg, blob, precision="fp32")
    d_frames = dev(frames)
    net = rh.enhance(d_frames)
    places, n = rh.identity_places(2)
    hr, sel = rh.unpack(net, places, n, d_frames, want_sel=True)
    o_net = oracle.sr_forward(cfg.net, blob, frames)
    o_hr, o_sel = oracle.unpack(frames, 2, o_net, oracle.identity_places(2, cfg.mbh, cfg.mbw))
    check_net(net.cpu().numpy(), o_net, "fp32", "frame-based cfg1")
    assert rel_l2(sel.cpu().numpy(), o_sel) <= 1e-5
    assert np.abs(hr.cpu().numpy().astype(int) - o_hr.astype(int)).max() <= 1
    rh.close()


# ---- bf16 / MFMA path --------------------------------------------------------------------

@pytest.mark.parametrize("net", [wl.Net("res", 32, 1, 2, 0.05), wl.Net("res", 64, 1, 2, 0.05),
                                 wl.Net("plain", 32, 3, 2, 0.05), wl.Net("plain", 64, 3, 4, 0.05),
                                 wl.Net("res", 32, 1, 3, 0.05), wl.Net("edsr", 64, 1, 2, 0.03),
                                 wl.Net("edsr", 64, 1, 3, 0.03), wl.Net("edsr", 64, 2, 4, 0.03),
                                 wl.Net("edsr", 32, 1, 4, 0.03)])
def test_small_topologies_bf16(net):
    """Small nets of every topology/scale/channel count the MFMA kernels serve; bins of 80 px
    give several 32-wide tiles with a ragged tail in both directions."""
    cfg = wl.replace(wl.config(1), net=net, n_frames=2, halo=5, frac=0.3, bin_size=80, precision="bf16")
    full_path_check(cfg)


@pytest.mark.parametrize("net", [wl.Net("edsr", 64, 1, 2, 0.03), wl.Net("edsr", 64, 1, 3, 0.03), wl.Net("edsr", 64, 2, 4, 0.03),
                                 wl.Net("edsr", 32, 1, 4, 0.03)])
def test_small_topologies_bf16_layer_by_layer_tail(net):
    """The same nets with the upsampler and the last conv run layer by layer (rh_config.per_layer_tail)
    instead of as one composed convolution."""
    cfg = wl.replace(wl.config(1), net=net, n_frames=2, halo=5, frac=0.3, bin_size=80, precision="bf16")
    full_path_check(cfg, per_layer_tail=True)


def test_cfg2_all_frames_bf16():
    full_path_check(wl.config(2))


def test_cfg3_two_frames_bf16():
    full_path_check(wl.config(3), n_frames=2)


def test_cfg3_two_frames_bf16_larger_output_amplitude():
    """The same net with a last conv 1.6 times larger (output rms 0.08, beyond the range the 2/255
    bar is claimed for): the error grows in proportion and the bar with it."""
    cfg = wl.config(3)
    full_path_check(wl.replace(cfg, net=wl.replace(cfg.net, tail_scale=0.02)), n_frames=2)


# ---- needed-region enhance mode (only pasted pixels matter, Sec. 3.3.3) ---------------------------

@pytest.mark.parametrize("net", [wl.Net("edsr", 64, 2, 2, 0.05), wl.Net("edsr", 64, 3, 4, 0.02), wl.Net("res", 64, 2, 2, 0.05),
                                 wl.Net("plain", 64, 4, 2, 0.05), wl.Net("edsr", 64, 2, 3, 0.05)],
                         ids=lambda n: f"{n.topology}x{n.scale}")
def test_needed_region_enhance_small_nets(net):
    full_path_check(wl.replace(wl.config(1), net=net, precision="bf16"), needed=True)


def test_needed_region_enhance_turned_boxes_and_odd_bin_side():
    cfg = wl.replace(wl.config(3), n_frames=2, width=160, height=112, halo=6, bin_size=88, importance="uniform", frac=0.4,
                     net=wl.Net("edsr", 64, 2, 4, 0.05))
    full_path_check(cfg, rotate=True, expect_turned=True, needed=True)


def test_needed_region_enhance_without_a_halo():
    """halo 0: pasted macroblocks touch the bin border, so the composed tail's border pass is needed too."""
    cfg = wl.replace(wl.config(1), net=wl.Net("edsr", 64, 2, 4, 0.02), precision="bf16", halo=0)
    full_path_check(cfg, needed=True)


def test_cfg3_two_frames_bf16_needed_region():
    full_path_check(wl.config(3), n_frames=2, needed=True)


@pytest.mark.parametrize("mode", ["needed", "masked"])
def test_list_modes_with_more_than_64_cells_per_bin(mode):
    """192 x 192 bins: 24 x 6 = 144 cells, so the list kernels go through a bin in three chunks of lanes."""
    cfg = wl.replace(wl.config(3), bin_size=192, net=wl.Net("edsr", 64, 2, 4, 0.02))
    full_path_check(cfg, n_frames=3, needed=mode == "needed", masked=mode == "masked")


def test_needed_region_enhance_rejects_the_layer_by_layer_tail():
    cfg = wl.replace(wl.config(3), n_frames=1, net=wl.Net("edsr", 64, 1, 4, 0.02))
    blob = wl.make_weights(cfg.net, 1, "bf16")
    rh = make_rh(cfg, blob, max_bins=4, per_layer_tail=True)
    bins = torch.zeros((1, cfg.bin_size, cfg.bin_size, 3), dtype=torch.uint8, device="cuda")
    places = torch.zeros((4, 16), dtype=torch.uint8, device="cuda")
    counts = torch.zeros(4, dtype=torch.int32, device="cuda")
    with pytest.raises(RuntimeError, match="per_layer_tail"):
        rh.enhance_needed(bins, places, counts)
    rh.close()


# ---- box-masked enhance mode (Sec. 3.3.2: bins are only partly occupied) -------------------------

@pytest.mark.parametrize("net", [wl.Net("edsr", 64, 2, 2, 0.05), wl.Net("edsr", 64, 1, 4, 0.02), wl.Net("res", 64, 2, 2, 0.05),
                                 wl.Net("plain", 64, 4, 2, 0.05), wl.Net("edsr", 64, 2, 3, 0.05)],
                         ids=lambda n: f"{n.topology}x{n.scale}")
def test_masked_enhance_small_nets(net):
    """320 x 192 frame, 64 x 64 bins (8 x 2 cells each), every topology of the 64-channel kernel."""
    full_path_check(wl.replace(wl.config(1), net=net, precision="bf16"), masked=True)


def test_masked_enhance_layer_by_layer_tail_and_odd_bin_side():
    """Bins of 80 x 80 pixels: 10 x 3 cells, the last column cut in half; upsampler run layer by layer."""
    cfg = wl.replace(wl.config(1), net=wl.Net("edsr", 64, 2, 4, 0.02), precision="bf16", bin_size=80)
    full_path_check(cfg, masked=True, per_layer_tail=True)


def test_cfg3_two_frames_bf16_masked():
    full_path_check(wl.config(3), n_frames=2, masked=True)


def test_masked_enhance_turned_boxes():
    """RotatePacking: a turned box marks the cells of its exchanged extent."""
    cfg = wl.replace(wl.config(3), n_frames=2, width=160, height=112, halo=6, bin_size=96, importance="uniform", frac=0.4,
                     net=wl.Net("edsr", 64, 2, 4, 0.05))
    full_path_check(cfg, rotate=True, expect_turned=True, masked=True)


def test_masked_enhance_without_boxes_is_the_tail_of_zero():
    """No box at all: every cell is cleared, the body computes nothing, and the layers after it
    run on a zero tensor; and a batch count of zero on the device writes nothing."""
    net = wl.Net("edsr", 64, 2, 4, 0.05)
    cfg = wl.replace(wl.config(3), net=net)
    blob = wl.make_weights(net, 2, "bf16")
    rh = make_rh(cfg, blob, max_bins=8)
    S = cfg.bin_size
    bins = torch.randint(0, 256, (2, S, S, 3), dtype=torch.uint8, device="cuda")
    boxes = torch.zeros((4, 24), dtype=torch.uint8, device="cuda")
    counts = torch.zeros(4, dtype=torch.int32, device="cuda")
    rh.enhance(bins)                                           # leaves other values in the workspace
    g = rh.enhance_masked(bins, boxes, counts).cpu().numpy()
    o = oracle.sr_forward(net, blob, bins.cpu().numpy(), np.zeros((2, S, S), dtype=np.uint8), body_only=True)
    check_net(g, o, "bf16", "masked, no boxes")
    out = torch.full((2, 4 * S, 4 * S, 3), 7.0, dtype=torch.float32, device="cuda")
    rh.enhance_masked(bins, boxes, counts, n_valid=counts[1:2], out=out)
    assert bool((out == 7.0).all())
    rh.close()


def test_masked_enhance_needs_the_64_channel_bf16_kernel():
    cfg = wl.config(1)
    blob = wl.make_weights(cfg.net, cfg.weight_seed, cfg.precision)
    rh = make_rh(cfg, blob)
    bins = torch.zeros((1, cfg.bin_size, cfg.bin_size, 3), dtype=torch.uint8, device="cuda")
    boxes = torch.zeros((4, 24), dtype=torch.uint8, device="cuda")
    counts = torch.zeros(4, dtype=torch.int32, device="cuda")
    with pytest.raises(RuntimeError, match="64 channels"):
        rh.enhance_masked(bins, boxes, counts)
    rh.close()


def test_frame_based_run_bf16_matches_oracle():
    cfg = wl.replace(wl.config(3), n_frames=1, width=112, height=80, net=wl.Net("edsr", 64, 3, 4, 0.02))
    frames = wl.make_frames(cfg)
    blob = wl.make_weights(cfg.net, 1, "bf16")
    rh = make_rh(cfg, blob)
    d_frames = dev(frames)
    net = rh.enhance(d_frames)
    places, n = rh.identity_places(1)
    hr, sel = rh.unpack(net, places, n, d_frames, want_sel=True)
    o_net = oracle.sr_forward(cfg.net, blob, frames)
    o_hr, o_sel = oracle.unpack(frames, 4, o_net, oracle.identity_places(1, cfg.mbh, cfg.mbw))
    check_net(net.cpu().numpy(), o_net, "bf16", "frame-based 112x80")
    assert rel_l2(sel.cpu().numpy(), o_sel) <= 1e-2 and np.abs(sel.cpu().numpy() - o_sel).max() <= 2 / 255
    assert np.abs(hr.cpu().numpy().astype(int) - o_hr.astype(int)).max() <= 2
    rh.close()


# ---- packing policy options (Alg. 1: Sort order, RotatePacking) ---------------------------------

@pytest.mark.parametrize("ci", [1, 3, 5])
@pytest.mark.parametrize("sort_policy,rotate", [("area", False), ("density", True), ("area", True)])
def test_policy_options_metadata_and_bytes_at_full_size(ci, sort_policy, rotate):
    cfg = wl.config(ci)
    frames, imp = wl.make_frames(cfg), wl.make_importance(cfg)
    net = wl.Net("plain", 4, 2, cfg.net.scale)
    blob = wl.make_weights(net, 0, "fp32")
    rh = make_rh(wl.replace(cfg, net=net), blob, precision="fp32", sort_policy=sort_policy, rotate=rotate)
    check_select_and_plan(rh, cfg, frames, imp, wl.make_segments(cfg), sort_policy=sort_policy, rotate=rotate)
    rh.close()


@pytest.mark.parametrize("seed", range(4))
def test_rotate_random_masks_metadata_and_bytes(seed):
    """Scattered selections in small bins: many boxes only fit turned."""
    cfg = wl.replace(wl.config(1), n_frames=4, width=160, height=112, halo=3 + seed, bin_size=64 + 16 * (seed % 3),
                     importance="uniform", frac=[0.2, 0.35, 0.5, 0.7][seed])
    frames, imp = wl.make_frames(cfg), wl.make_importance(cfg)
    net = wl.Net("plain", 4, 2, 2)
    rh = make_rh(wl.replace(cfg, net=net), wl.make_weights(net, 0, "fp32"), precision="fp32", rotate=True,
                 connectivity=4 if seed % 2 else 8)
    o_plan, *_ = check_select_and_plan(rh, cfg, frames, imp, wl.make_segments(cfg), conn=4 if seed % 2 else 8, rotate=True)
    assert o_plan.boxes[:, 5].sum() > 0
    rh.close()


def test_rotate_whole_path_fp32():
    cfg = wl.replace(wl.config(1), n_frames=3, width=160, height=112, halo=4, bin_size=64, importance="uniform", frac=0.5)
    full_path_check(cfg, rotate=True, expect_turned=True)


@pytest.mark.parametrize("scale", [3, 4])
def test_rotate_whole_path_bf16_edsr(scale):
    cfg = wl.replace(wl.config(3), n_frames=2, width=160, height=112, halo=6, bin_size=96, importance="uniform", frac=0.4,
                     net=wl.Net("edsr", 64, 2, scale, 0.05))
    full_path_check(cfg, rotate=True, expect_turned=True)


# ---- full benchmark sizes, in the launch configuration bench.py times --------------------------

@pytest.mark.timeout(600)
@pytest.mark.parametrize("ci,sample", [(3, None), (5, 8)])
def test_full_size_bf16(ci, sample):
    """The whole batch of configurations 3 and 5 through the path exactly as bench.py drives it
    (capacity-sized enhance call with the device-side bin count).  Metadata and packed bytes are
    compared in full.  Configuration 3: the network output of ALL bins and the pasted pixels of ALL
    selected macroblocks, element by element.  Configuration 5: the same on 8 bins spread over the
    batch.  Every unselected macroblock of every frame against the bilinear base, and bins past the
    count must stay untouched."""
    cfg = wl.config(ci)
    F, s, S = cfg.n_frames, cfg.net.scale, cfg.bin_size
    frames, imp, segs = wl.make_frames(cfg), wl.make_importance(cfg), wl.make_segments(cfg)
    blob = wl.make_weights(cfg.net, cfg.weight_seed, cfg.precision)
    max_bins = 512 if ci == 5 else 256
    rh = make_rh(cfg, blob, max_bins=max_bins)
    o_plan, po, (d_frames, d_imp, o_bins) = check_select_and_plan(rh, cfg, frames, imp, segs, max_bins=max_bins)
    nb = o_plan.n_bins
    net_out = torch.full((nb + 1, S * s, S * s, 3), 7.0, dtype=torch.float32, device="cuda")
    # capacity (nb + 1 images) above the device-side count (nb): the last image must not be touched
    rh.enhance(po.bins[: nb + 1], n=nb + 1, n_valid=po.counts[1:2], out=net_out)
    assert bool((net_out[nb] == 7.0).all()), "an image past the device-side count was written"
    hr, sel = rh.unpack(net_out, po.places, po.counts[3:4], d_frames, want_sel=True)
    pick = list(range(nb)) if sample is None else sorted({int(round(i * (nb - 1) / (sample - 1))) for i in range(sample)})
    print(f"[{cfg.name}] {nb} bins, oracle on {len(pick)} of them", flush=True)
    o_net = oracle.sr_forward(cfg.net, blob, o_bins[pick])
    check_net(net_out[pick].cpu().numpy(), o_net, "bf16", f"{cfg.name} {len(pick)} of {nb} bins")
    bar = bf16_max_abs_bar(o_net)
    assert bar == 2.0 / 255.0, "the benchmark nets stay inside the output range the 2/255 bar is claimed for"
    # pasted pixels of the macroblocks that live in the checked bins
    B = 16 * s
    g_sel = sel.cpu().numpy()
    per = cfg.mbw * cfg.mbh
    worst, n_chk = 0.0, 0
    base_cache = {}
    where = {b: i for i, b in enumerate(pick)}
    for i, (g, box, b, px, py) in enumerate(o_plan.places.tolist()):
        if b not in where:
            continue
        f, rem = divmod(g, per); y, x = divmod(rem, cfg.mbw)
        if f not in base_cache:
            base_cache[f] = oracle.bilinear(frames[f], s)
        base = base_cache[f][y * B:(y + 1) * B, x * B:(x + 1) * B].astype(np.float32) / np.float32(255.0)
        blk = o_net[where[b], py * s:py * s + B, px * s:px * s + B].astype(np.float32)
        want = np.clip(base + blk, 0.0, 1.0)
        worst = max(worst, float(np.abs(g_sel[i] - want).max())); n_chk += 1
    print(f"[{cfg.name}] {n_chk} of {len(o_plan.places)} pasted macroblocks checked, max abs={worst:.3e} (bar {bar:.3e})", flush=True)
    assert n_chk > 0 and worst <= bar
    if sample is None:
        assert n_chk == len(o_plan.places)
    # every unselected macroblock of every frame is the bilinear base, byte for byte
    g_hr = hr.cpu().numpy()
    o_mask = oracle.select(imp, segs)[0]
    for f in range(F):
        base = base_cache.get(f)
        if base is None:
            base = oracle.bilinear(frames[f], s)
        keep = ~np.kron(o_mask[f], np.ones((B, B), dtype=np.uint8)).astype(bool)
        assert np.array_equal(g_hr[f][keep], base[keep])
    rh.close()


@pytest.mark.parametrize("ci", [3, 5])
def test_full_size_needed_region_pastes_the_same_frames(ci):
    """Configurations 3 and 5 in the launch configuration bench.py times (capacity-sized call, device-side
    bin count): the needed-region mode's pasted frames and enhanced pixels equal the plain mode's bit for
    bit (the plain mode's are compared with the oracle in test_full_size_bf16), whatever the workspace
    and the output buffer held before."""
    cfg = wl.config(ci)
    s, S = cfg.net.scale, cfg.bin_size
    frames, imp, segs = wl.make_frames(cfg), wl.make_importance(cfg), wl.make_segments(cfg)
    blob = wl.make_weights(cfg.net, cfg.weight_seed, cfg.precision)
    max_bins = 512 if ci == 5 else 256
    rh = make_rh(cfg, blob, max_bins=max_bins)
    d_frames, d_imp = dev(frames), dev(imp)
    seg_rows = [tuple(r) for r in np.asarray(segs).tolist()]
    mask, lst, n_sel = rh.select_regions(d_imp, seg_rows)
    po = rh.pack(d_frames, d_imp, mask, lst, n_sel)
    nb = int(po.counts[1])
    cap = nb + 3
    net = torch.empty((cap, S * s, S * s, 3), dtype=torch.float32, device="cuda")
    rh.enhance(po.bins[:cap], n=cap, n_valid=po.counts[1:2], out=net)
    hr0, sel0 = rh.unpack(net, po.places, po.counts[3:4], d_frames, want_sel=True)
    net.fill_(float("nan"))
    rh.enhance_needed(po.bins[:cap], po.places, po.counts, n=cap, n_valid=po.counts[1:2], out=net)
    hr1, sel1 = rh.unpack(net, po.places, po.counts[3:4], d_frames, want_sel=True)
    k = int(po.counts[3])
    assert k > 1000 and torch.equal(sel0[:k], sel1[:k]) and torch.equal(hr0, hr1)
    assert not bool(torch.isnan(sel1[:k]).any())
    written = float((~torch.isnan(net[:nb])).float().mean())
    print(f"[{cfg.name}] needed-region mode wrote {written:.3f} of the bins' output pixels", flush=True)
    assert written < 0.9                                       # the tail really skipped what is not pasted
    rh.close()


@pytest.mark.timeout(300)
def test_frame_based_run_bf16_full_size_frames():
    """The 100 % run of the fraction sweep at its real shape: whole 480 x 272 frames through rh_enhance
    and the identity placement, two frames of the batch against the oracle element by element."""
    cfg = wl.config(4)
    F, s = 2, cfg.net.scale
    frames = wl.make_frames(cfg, F)
    blob = wl.make_weights(cfg.net, cfg.weight_seed, "bf16")
    rh = make_rh(cfg, blob, n_frames=F, max_bins=4)
    d_frames = dev(frames)
    net = rh.enhance(d_frames)
    places, n = rh.identity_places(F)
    hr, sel = rh.unpack(net, places, n, d_frames, want_sel=True)
    o_net = oracle.sr_forward(cfg.net, blob, frames)
    o_hr, o_sel = oracle.unpack(frames, s, o_net, oracle.identity_places(F, cfg.mbh, cfg.mbw))
    check_net(net.cpu().numpy(), o_net, "bf16", "frame-based 2 x 480x272")
    d = np.abs(sel.cpu().numpy() - o_sel)
    print(f"[frame-based 2 x 480x272] pasted pixels max abs={d.max():.3e}", flush=True)
    assert d.max() <= bf16_max_abs_bar(o_net) == 2.0 / 255.0
    assert np.abs(hr.cpu().numpy().astype(int) - o_hr.astype(int)).max() <= 2
    rh.close()


# ---- exact-border mode ---------------------------------------------------------------------------

def exact_border_check(cfg, precision, rotate=False, border_bias=True):
    F, s = cfg.n_frames, cfg.net.scale
    frames, imp, segs = wl.make_frames(cfg), wl.make_importance(cfg), wl.make_segments(cfg)
    if border_bias:                                           # pull border macroblocks into the selection
        imp[:, 0, :] += 5.0; imp[:, :, 0] += 5.0; imp[:, -1, -3:] += 5.0
    blob = wl.make_weights(cfg.net, cfg.weight_seed, precision)
    rh = make_rh(cfg, blob, precision=precision, rotate=rotate)
    o_plan, po, (d_frames, d_imp, o_bins) = check_select_and_plan(rh, cfg, frames, imp, segs, rotate=rotate)
    keep = oracle.border_keep(cfg.height, cfg.width, o_plan.boxes, cfg.halo, cfg.bin_size, o_plan.n_bins)
    assert (keep == 0).sum() > 0
    o_net = oracle.sr_forward(cfg.net, blob, o_bins, keep)
    o_plain = oracle.sr_forward(cfg.net, blob, o_bins)
    g_net = rh.enhance_exact(po.bins, po.boxes, po.counts, n=o_plan.n_bins, n_valid=po.counts[1:2]).cpu().numpy()
    tol = 1e-5 if precision == "fp32" else 1e-2
    e, _ = check_net(g_net, o_net, precision, f"{cfg.name} exact-border")
    e_plain = rel_l2(g_net, o_plain)
    print(f"[{cfg.name}/{precision}] exact-border against the plain mode: {e_plain:.3e}", flush=True)
    assert e <= tol and e_plain > 3 * e
    # the plain call is unchanged by the exact one having run
    g_plain = rh.enhance(po.bins, n=o_plan.n_bins).cpu().numpy()
    check_net(g_plain, o_plain, precision, f"{cfg.name} plain after exact")
    rh.close()
    return g_net, o_plan, frames, blob


def test_exact_border_fp32_equals_frame_based_at_border_macroblocks():
    """fp32, halo = receptive-field radius: the GPU's exact-border output equals the GPU-independent
    whole-frame oracle run at every selected macroblock, border ones included."""
    cfg = wl.config(1)
    g_net, o_plan, frames, blob = exact_border_check(cfg, "fp32")
    s, B = cfg.net.scale, 16 * cfg.net.scale
    full = oracle.sr_forward(cfg.net, blob, frames)[0]
    worst = 0.0
    for g, box, b, px, py in o_plan.places.tolist():
        y, x = divmod(g, cfg.mbw)
        worst = max(worst, float(np.abs(g_net[b, py * s:py * s + B, px * s:px * s + B] - full[y * B:(y + 1) * B, x * B:(x + 1) * B]).max()))
    assert worst <= 1e-5, worst


@pytest.mark.parametrize("net", [wl.Net("edsr", 8, 2, 4, 0.05), wl.Net("res", 8, 2, 2, 0.05), wl.Net("edsr", 12, 1, 3, 0.05)])
def test_exact_border_fp32_topologies_with_turned_boxes(net):
    cfg = wl.replace(wl.config(1), net=net, n_frames=3, width=160, height=112, halo=4, bin_size=64, importance="uniform", frac=0.5)
    exact_border_check(cfg, "fp32", rotate=True)


@pytest.mark.parametrize("net", [wl.Net("edsr", 64, 2, 4, 0.02), wl.Net("edsr", 64, 1, 3, 0.02), wl.Net("res", 32, 2, 2, 0.03)])
def test_exact_border_bf16(net):
    cfg = wl.replace(wl.config(3), n_frames=2, width=160, height=112, halo=6, bin_size=96, net=net)
    exact_border_check(cfg, "bf16")


# ---- frame sides that are not multiples of 16 ----------------------------------------------------

@pytest.mark.parametrize("w,h,net,precision", [
    (168, 100, wl.Net("plain", 16, 4, 2, 0.1), "fp32"),
    (170, 90, wl.Net("edsr", 8, 1, 3, 0.05), "fp32"),          # row pitch of the output not a multiple of 4 bytes
    (200, 120, wl.Net("edsr", 64, 2, 4, 0.02), "bf16"),
])
def test_partial_macroblock_frames_whole_path(w, h, net, precision):
    cfg = wl.replace(wl.config(1), width=w, height=h, n_frames=2, net=net, halo=5, bin_size=96, frac=0.3, precision=precision)
    F = 2
    frames, imp = wl.make_frames(cfg), wl.make_importance(cfg)
    imp[:, -1, :] += 5.0; imp[:, :, -1] += 5.0                 # the cut macroblocks at the right and bottom edges
    k = int(imp.size * 0.3)
    segs = np.array([[0, F, k]], dtype=np.uint32)
    blob = wl.make_weights(cfg.net, 0, precision)
    rh = make_rh(cfg, blob, precision=precision)
    o_plan, po, (d_frames, d_imp, o_bins) = check_select_and_plan(rh, cfg, frames, imp, segs)
    s = cfg.net.scale
    g_net = rh.enhance(po.bins, n=o_plan.n_bins)
    o_net = oracle.sr_forward(cfg.net, blob, o_bins)
    tol = 1e-5 if precision == "fp32" else 1e-2
    check_net(g_net.cpu().numpy(), o_net, precision, f"partial {w}x{h}")
    sel0 = torch.full((po.places.shape[0], 16 * s, 16 * s, 3), 9.0, dtype=torch.float32, device="cuda")   # stale values must be overwritten
    hr, sel = rh.unpack(g_net, po.places, po.counts[3:4], d_frames, want_sel=True, sel=sel0)
    o_hr, o_sel = oracle.unpack(frames, s, o_net, o_plan.places)
    assert hr.shape == (F, h * s, w * s, 3)
    g_sel = sel[: len(o_plan.places)].cpu().numpy()
    assert rel_l2(g_sel, o_sel) <= tol
    per = cfg.mbw * cfg.mbh
    for i, (g, box, b, px, py) in enumerate(o_plan.places.tolist()):     # the outside part of a cut block must read 0
        y, x = divmod(g % per, cfg.mbw)
        h_in, w_in = min(16, h - 16 * y) * s, min(16, w - 16 * x) * s
        assert not g_sel[i, h_in:].any() and not g_sel[i, :, w_in:].any()
    d = np.abs(hr.cpu().numpy().astype(np.int16) - o_hr.astype(np.int16))
    B = 16 * s
    selmask = np.kron(oracle.select(imp, segs)[0], np.ones((B, B), dtype=np.uint8)).astype(bool)[:, :h * s, :w * s]
    assert d[~selmask].max() == 0
    assert d.max() <= (1 if precision == "fp32" else 2)
    # frame-based run on the same frames: identity placement with cut blocks at the edges
    f_net = rh.enhance(d_frames)
    places, n = rh.identity_places(F)
    hr2, sel2 = rh.unpack(f_net, places, n, d_frames, want_sel=True)
    of_net = oracle.sr_forward(cfg.net, blob, frames)
    o_hr2, o_sel2 = oracle.unpack(frames, s, of_net, oracle.identity_places(F, cfg.mbh, cfg.mbw))
    check_net(f_net.cpu().numpy(), of_net, precision, f"partial {w}x{h} frame-based")
    assert rel_l2(sel2.cpu().numpy(), o_sel2) <= tol
    assert np.abs(hr2.cpu().numpy().astype(np.int16) - o_hr2.astype(np.int16)).max() <= (1 if precision == "fp32" else 2)
    rh.close()


# ---- rh_enhance on odd image shapes ----------------------------------------------------------------

@pytest.mark.parametrize("precision,net", [("bf16", wl.Net("edsr", 64, 1, 4, 0.02)), ("bf16", wl.Net("edsr", 64, 1, 3, 0.02)),
                                           ("bf16", wl.Net("res", 32, 1, 2, 0.03)), ("fp32", wl.Net("edsr", 8, 1, 2, 0.05))])
def test_enhance_small_and_ragged_images(precision, net):
    """rh_enhance takes any H, W >= 3: images smaller than one tile, one pixel over a tile edge, prime sizes."""
    cfg = wl.replace(wl.config(1), net=net, precision=precision)
    blob = wl.make_weights(net, 3, precision)
    rh = make_rh(cfg, blob, precision=precision)
    rng = np.random.default_rng(11)
    tol = 1e-5 if precision == "fp32" else 1e-2
    for (n, h, w) in [(2, 3, 3), (1, 5, 7), (3, 17, 33), (1, 16, 32), (2, 31, 65), (1, 9, 130)]:
        imgs = rng.integers(0, 256, size=(n, h, w, 3), dtype=np.uint8)
        got = rh.enhance(dev(imgs)).cpu().numpy()
        want = oracle.sr_forward(net, blob, imgs)
        assert got.shape == want.shape
        check_net(got, want, precision, f"{net.topology}{net.channels}x{net.scale} {n}x{h}x{w}")
    rh.close()
