"""Pins for the oracle's pixel steps: closed forms, brute force in exact rationals, and
library routines (torch on CPU, fp64) as a second opinion, plus the invariants that tie the
packed path to frame-based SR (Sec. 3.2.1 problem statement, Sec. 3.3.3)."""
from fractions import Fraction

import numpy as np
import pytest
import torch
import torch.nn.functional as TF

import workloads as wl


def t_conv(x, w, b):
    """library second opinion: x [H,W,Cin] fp64, w [Cout,3,3,Cin], b [Cout]."""
    xt = torch.from_numpy(np.ascontiguousarray(x)).permute(2, 0, 1)[None].double()
    wt = torch.from_numpy(np.ascontiguousarray(w)).permute(0, 3, 1, 2).double()
    y = TF.conv2d(xt, wt, torch.from_numpy(b).double(), padding=1)
    return y[0].permute(1, 2, 0).numpy()


def test_conv_delta_kernels_shift(orc):
    rng = np.random.default_rng(0)
    x = rng.standard_normal((7, 9, 3))
    for ky in range(3):
        for kx in range(3):
            w = np.zeros((3, 3, 3, 3), dtype=np.float32)
            for c in range(3):
                w[c, ky, kx, c] = 1.0
            y = orc.conv3x3(x, w, np.zeros(3, dtype=np.float32))
            want = np.zeros_like(x)
            for yy in range(7):
                for xx in range(9):
                    sy, sx = yy + ky - 1, xx + kx - 1
                    if 0 <= sy < 7 and 0 <= sx < 9:
                        want[yy, xx] = x[sy, sx]
            assert np.array_equal(y, want)


def test_conv_vs_library_linearity_bias_relu(orc):
    rng = np.random.default_rng(1)
    x = rng.standard_normal((11, 6, 5)); x2 = rng.standard_normal((11, 6, 5))
    w = rng.standard_normal((4, 3, 3, 5)).astype(np.float32)
    b = rng.standard_normal(4).astype(np.float32)
    y = orc.conv3x3(x, w, b)
    assert np.allclose(y, t_conv(x, w, b), rtol=1e-12, atol=1e-12)
    zero = np.zeros(4, dtype=np.float32)
    lin = orc.conv3x3(2.0 * x + x2, w, zero)
    assert np.allclose(lin, 2.0 * orc.conv3x3(x, w, zero) + orc.conv3x3(x2, w, zero), atol=1e-12)
    assert np.allclose(orc.conv3x3(np.zeros_like(x), w, b), np.broadcast_to(b.astype(np.float64), y.shape))
    assert np.array_equal(orc.conv3x3(x, w, b, relu=True), np.maximum(y, 0.0))
    # translation equivariance away from the border
    xs = np.roll(x, (2, 1), axis=(0, 1))
    ys = orc.conv3x3(xs, w, b)
    assert np.allclose(ys[4:-1, 3:-1], y[2:-3, 2:-2], atol=1e-12)


def test_pixel_shuffle_vs_library_and_definition(orc):
    rng = np.random.default_rng(2)
    for r in (2, 3):
        x = rng.standard_normal((4, 5, 3 * r * r))
        y = orc.pixel_shuffle(x, r)
        lib = TF.pixel_shuffle(torch.from_numpy(x).permute(2, 0, 1)[None], r)[0].permute(1, 2, 0).numpy()
        assert np.array_equal(y, lib)
        assert y[1 * r + (r - 1), 2 * r + 1, 2] == x[1, 2, 2 * r * r + (r - 1) * r + 1]


def bilinear_exact(img, s):
    H, W, _ = img.shape
    out = np.zeros((H * s, W * s, 3), dtype=np.uint8)
    for Y in range(H * s):
        sy = Fraction(2 * Y + 1, 2 * s) - Fraction(1, 2)
        y0 = sy.numerator // sy.denominator; fy = sy - y0
        for X in range(W * s):
            sx = Fraction(2 * X + 1, 2 * s) - Fraction(1, 2)
            x0 = sx.numerator // sx.denominator; fx = sx - x0
            for c in range(3):
                def p(y, x):
                    return int(img[min(max(y, 0), H - 1), min(max(x, 0), W - 1), c])
                v = ((1 - fy) * ((1 - fx) * p(y0, x0) + fx * p(y0, x0 + 1))
                     + fy * ((1 - fx) * p(y0 + 1, x0) + fx * p(y0 + 1, x0 + 1)))
                q = v + Fraction(1, 2)
                out[Y, X, c] = q.numerator // q.denominator          # round half up
    return out


def test_bilinear_closed_forms_and_exact_rationals(orc):
    rng = np.random.default_rng(3)
    img = rng.integers(0, 256, size=(5, 6, 3), dtype=np.uint8)
    assert np.array_equal(orc.bilinear(img, 1), img)
    const = np.full((4, 4, 3), 77, dtype=np.uint8)
    for s in (2, 3, 4):
        assert np.all(orc.bilinear(const, s) == 77)
        got = orc.bilinear(img, s)
        assert np.array_equal(got, bilinear_exact(img, s))
        lib = TF.interpolate(torch.from_numpy(img).permute(2, 0, 1)[None].double(), scale_factor=s,
                             mode="bilinear", align_corners=False)[0].permute(1, 2, 0).numpy()
        assert np.abs(got.astype(np.float64) - lib).max() <= 0.5 + 1e-9


def test_gather_bytes(orc):
    cfg = wl.replace(wl.config(1), n_frames=2)
    frames = wl.make_frames(cfg)
    imp = wl.make_importance(cfg)
    mask, lst = orc.select(imp, np.array([[0, 2, 150]], dtype=np.uint32))
    pl = orc.plan(mask, imp, cfg.halo, cfg.bin_size)
    bins = orc.gather(frames, pl.boxes, cfg.halo, cfg.bin_size, pl.n_bins)
    covered = np.zeros(bins.shape[:3], dtype=bool)
    H, W = cfg.height, cfg.width
    for (f, x0, y0, w, h, rot, b, bx, by, bid) in pl.boxes.tolist():
        bw, bh = 16 * w + 2 * cfg.halo, 16 * h + 2 * cfg.halo
        src = np.zeros((bh, bw, 3), dtype=np.uint8)
        ys = np.arange(16 * y0 - cfg.halo, 16 * y0 - cfg.halo + bh); xs = np.arange(16 * x0 - cfg.halo, 16 * x0 - cfg.halo + bw)
        vy = (ys >= 0) & (ys < H); vx = (xs >= 0) & (xs < W)
        src[np.ix_(vy, vx)] = frames[f][np.ix_(ys[vy], xs[vx])]
        assert np.array_equal(bins[b, by:by + bh, bx:bx + bw], src)
        assert not covered[b, by:by + bh, bx:bx + bw].any()
        covered[b, by:by + bh, bx:bx + bw] = True
    assert np.all(bins[~covered] == 0)
    for g, box, b, px, py in pl.places.tolist():        # every owned MB sits where its row says
        f, rem = divmod(g, cfg.mbw * cfg.mbh); y, x = divmod(rem, cfg.mbw)
        assert np.array_equal(bins[b, py:py + 16, px:px + 16], frames[f, 16 * y:16 * y + 16, 16 * x:16 * x + 16])


def t_net(net, blob, img):
    """The three topologies composed from library ops (fp64), as a second opinion."""
    x = torch.from_numpy(img.astype(np.float64) / 255.0).permute(2, 0, 1)[None]
    pos = 0
    layers = []
    for cin, cout, _ in wl.net_layers(net):
        w = torch.from_numpy(blob[pos:pos + cout * 9 * cin].reshape(cout, 3, 3, cin)).permute(0, 3, 1, 2).double(); pos += cout * 9 * cin
        b = torch.from_numpy(blob[pos:pos + cout]).double(); pos += cout
        layers.append((w, b))
    assert pos == len(blob)
    it = iter(layers)
    conv = lambda t: TF.conv2d(t, *next(it), padding=1)
    if net.topology == "plain":
        for _ in range(net.n_blocks - 1):
            x = torch.relu(conv(x))
        y = TF.pixel_shuffle(conv(x), net.scale)
    else:
        x = conv(x); head = x
        for _ in range(net.n_blocks):
            x = x + conv(torch.relu(conv(x)))
        if net.topology == "res":
            y = TF.pixel_shuffle(conv(x), net.scale)
        else:
            x = conv(x) + head
            for _ in range(2 if net.scale == 4 else 1):
                x = TF.pixel_shuffle(conv(x), 2 if net.scale == 4 else net.scale)
            y = conv(x)
    return y[0].permute(1, 2, 0).numpy()


@pytest.mark.parametrize("net", [wl.Net("plain", 8, 4, 2), wl.Net("res", 8, 3, 2), wl.Net("res", 4, 2, 3),
                                 wl.Net("edsr", 8, 2, 2), wl.Net("edsr", 8, 2, 3), wl.Net("edsr", 8, 3, 4)])
def test_sr_forward_vs_library_composition(orc, net):
    rng = np.random.default_rng(5)
    blob = wl.make_weights(net, 3, "fp32")
    imgs = rng.integers(0, 256, size=(2, 9, 7, 3), dtype=np.uint8)
    out = orc.sr_forward(net, blob, imgs)
    for n in range(2):
        want = t_net(net, blob, imgs[n])
        assert out[n].shape == want.shape
        assert np.allclose(out[n], want, rtol=1e-11, atol=1e-11)
    assert out.std() > 1e-3


def test_weight_blob_bf16_exact_and_sizes():
    for ci in (1, 2, 3, 5):
        cfg = wl.config(ci)
        blob = wl.make_weights(cfg.net, cfg.weight_seed, cfg.precision)
        assert len(blob) == sum(co * 9 * ci_ + co for ci_, co, _ in wl.net_layers(cfg.net))
        if cfg.precision == "bf16":
            assert np.all(blob.view(np.uint32) & 0xFFFF == 0)
    x = np.array([1.0, 1.00390625, 1.0078125 + 2 ** -8, -3.14159, 1e-40], dtype=np.float32)
    r = wl.round_to_bf16(x)
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == np.float32(1.015625)   # ties go to the even mantissa
    assert torch.equal(torch.from_numpy(r), torch.from_numpy(x).bfloat16().float())


# --- whole-path invariants ---------------------------------------------------------------

def test_unselected_is_exactly_bilinear_and_paste_formula(orc):
    cfg = wl.config(1)
    frames, imp = wl.make_frames(cfg), wl.make_importance(cfg)
    blob = wl.make_weights(cfg.net, cfg.weight_seed, cfg.precision)
    r = orc.run_path(frames, imp, wl.make_segments(cfg), cfg.net, blob, cfg.halo, cfg.bin_size)
    s = cfg.net.scale
    base = orc.bilinear(frames[0], s)
    B = 16 * s
    changed = 0
    for y in range(cfg.mbh):
        for x in range(cfg.mbw):
            blk = r.frames_hr[0, y * B:(y + 1) * B, x * B:(x + 1) * B]
            bb = base[y * B:(y + 1) * B, x * B:(x + 1) * B]
            if not r.mask[0, y, x]:
                assert np.array_equal(blk, bb)
            else:
                changed += int((blk != bb).any())
    assert changed == 60
    # paste = clamp(base/255 + net) at the placed position, quantised round-half-up
    for i, (g, box, b, px, py) in enumerate(r.plan.places.tolist()):
        y, x = divmod(g, cfg.mbw)
        net = r.net_out[b, py * s:py * s + B, px * s:px * s + B]
        e = np.clip(base[y * B:(y + 1) * B, x * B:(x + 1) * B].astype(np.float64) / 255.0 + net, 0, 1)
        assert np.abs(r.sel[i] - e).max() < 1e-6
        q = np.floor(e * 255.0 + 0.5)
        got = r.frames_hr[0, y * B:(y + 1) * B, x * B:(x + 1) * B].astype(np.float64)
        assert np.abs(got - q).max() <= 1 and (got != q).mean() < 1e-3
    assert 0.005 < r.net_out.std() < 0.5 and (r.sel > 0).mean() > 0.9 and (r.sel < 1).mean() > 0.9


def test_halo_ge_receptive_field_equals_frame_based(orc):
    """cfg 1: 4 convs -> receptive-field radius 4 = halo.  The packed path then equals SR of the
    frame on a zero canvas at every selected MB, and plain frame-based SR at selected MBs that lie
    at least 4 px away from the frame border."""
    cfg = wl.config(1)
    frames, imp = wl.make_frames(cfg), wl.make_importance(cfg)
    blob = wl.make_weights(cfg.net, cfg.weight_seed, cfg.precision)
    r = orc.run_path(frames, imp, wl.make_segments(cfg), cfg.net, blob, cfg.halo, cfg.bin_size)
    s, R, B = cfg.net.scale, 4, 16 * cfg.net.scale
    canvas = np.zeros((1, cfg.height + 2 * R, cfg.width + 2 * R, 3), dtype=np.uint8)
    canvas[0, R:-R, R:-R] = frames[0]
    full_canvas = orc.sr_forward(cfg.net, blob, canvas)[0][R * s:-R * s, R * s:-R * s]
    full_plain = orc.sr_forward(cfg.net, blob, frames)[0]
    n_interior = 0
    for g, box, b, px, py in r.plan.places.tolist():
        y, x = divmod(g, cfg.mbw)
        packed = r.net_out[b, py * s:py * s + B, px * s:px * s + B]
        assert np.array_equal(packed, full_canvas[y * B:(y + 1) * B, x * B:(x + 1) * B])
        if 0 < y < cfg.mbh - 1 and 0 < x < cfg.mbw - 1:
            n_interior += 1
            assert np.array_equal(packed, full_plain[y * B:(y + 1) * B, x * B:(x + 1) * B])
    assert n_interior >= 20
    # and with a halo one pixel short of R the equality must break somewhere
    r3 = orc.run_path(frames, imp, wl.make_segments(cfg), cfg.net, blob, 3, cfg.bin_size)
    diff = 0
    for g, box, b, px, py in r3.plan.places.tolist():
        y, x = divmod(g, cfg.mbw)
        diff += not np.array_equal(r3.net_out[b, py * s:py * s + B, px * s:px * s + B],
                                   full_canvas[y * B:(y + 1) * B, x * B:(x + 1) * B])
    assert diff > 0


def test_all_selected_single_bin_equals_frame_based(orc):
    """A 48x48 frame, everything selected, halo 4 = R, bin 64: one box, and the pasted result is
    the frame-based run on the zero canvas; the identity placement reproduces it too."""
    cfg = wl.replace(wl.config(1), width=48, height=48)
    frames = wl.make_frames(cfg)
    imp = wl.make_importance(cfg)
    blob = wl.make_weights(cfg.net, 0, "fp32")
    r = orc.run_path(frames, imp, np.array([[0, 1, 9]], dtype=np.uint32), cfg.net, blob, 4, 64)
    assert r.plan.n_bins == 1 and len(r.plan.boxes) == 1
    canvas = np.zeros((1, 56, 56, 3), dtype=np.uint8); canvas[0, 4:-4, 4:-4] = frames[0]
    net = orc.sr_forward(cfg.net, blob, canvas)
    pl = orc.identity_places(1, 3, 3); pl[:, 3:] += 4
    hr, sel = orc.unpack(frames, 2, net, pl)
    assert np.array_equal(hr, r.frames_hr) and np.array_equal(sel, r.sel)


def _rotating_case(orc):
    """A small batch whose plan turns at least one box when RotatePacking is on."""
    rng = np.random.default_rng(7)
    F, mbh, mbw = 3, 6, 8
    cfg = wl.replace(wl.config(1), n_frames=F, width=16 * mbw, height=16 * mbh)
    frames = wl.make_frames(cfg)
    mask = (rng.random((F, mbh, mbw)) < 0.35).astype(np.uint8)
    imp = rng.random((F, mbh, mbw)).astype(np.float32)
    pl = orc.plan(mask, imp, 4, 80, 4, 4, rotate=True)
    assert pl.boxes[:, 5].sum() > 0 and (pl.boxes[:, 3] != pl.boxes[:, 4])[pl.boxes[:, 5] == 1].all()
    return cfg, frames, mask, imp, pl


def test_gather_turned_boxes_are_transposed_windows(orc):
    """Alg. 1, RotatePacking: a turned box is the transposed source window (numpy's transpose is
    the definition here), upright boxes are the window itself, everything else is zero."""
    cfg, frames, mask, imp, pl = _rotating_case(orc)
    halo, S, H, W = 4, 80, cfg.height, cfg.width
    bins = orc.gather(frames, pl.boxes, halo, S, pl.n_bins)
    covered = np.zeros(bins.shape[:3], dtype=bool)
    for (f, x0, y0, w, h, rot, b, bx, by, bid) in pl.boxes.tolist():
        bw, bh = 16 * w + 2 * halo, 16 * h + 2 * halo
        src = np.zeros((bh, bw, 3), dtype=np.uint8)
        ys = np.arange(16 * y0 - halo, 16 * y0 - halo + bh); xs = np.arange(16 * x0 - halo, 16 * x0 - halo + bw)
        vy = (ys >= 0) & (ys < H); vx = (xs >= 0) & (xs < W)
        src[np.ix_(vy, vx)] = frames[f][np.ix_(ys[vy], xs[vx])]
        if rot:
            src = src.transpose(1, 0, 2); bw, bh = bh, bw
        assert np.array_equal(bins[b, by:by + bh, bx:bx + bw], src)
        assert not covered[b, by:by + bh, bx:bx + bw].any()
        covered[b, by:by + bh, bx:bx + bw] = True
    assert np.all(bins[~covered] == 0)
    for (g, box, b, px, py), rot in zip(pl.places.tolist(), pl.place_rot.tolist()):
        f, rem = divmod(g, cfg.mbw * cfg.mbh); y, x = divmod(rem, cfg.mbw)
        mb = frames[f, 16 * y:16 * y + 16, 16 * x:16 * x + 16]
        assert np.array_equal(bins[b, py:py + 16, px:px + 16], mb.transpose(1, 0, 2) if rot else mb)


def test_paste_turned_boxes_transposes_back(orc):
    """The paste of a turned box reads the enhanced block transposed: with an 'enhancer' whose output
    is a known function of the bin coordinates, every pasted value is checked against that function
    at the exchanged coordinates, in numpy."""
    cfg, frames, mask, imp, pl = _rotating_case(orc)
    s, S = 2, 80
    B = 16 * s
    rng = np.random.default_rng(3)
    net = rng.uniform(-0.2, 0.2, size=(pl.n_bins, S * s, S * s, 3))
    hr, sel = orc.unpack(frames, s, net, pl.places, place_rot=pl.place_rot)
    n_rot = 0
    for i, ((g, box, b, px, py), rot) in enumerate(zip(pl.places.tolist(), pl.place_rot.tolist())):
        f, rem = divmod(g, cfg.mbw * cfg.mbh); y, x = divmod(rem, cfg.mbw)
        blk = net[b, py * s:py * s + B, px * s:px * s + B]
        if rot:
            blk = blk.transpose(1, 0, 2); n_rot += 1
        base = orc.bilinear(frames[f], s)[y * B:(y + 1) * B, x * B:(x + 1) * B].astype(np.float64) / 255.0
        e = np.clip(base + blk, 0, 1)
        assert np.abs(sel[i] - e).max() < 1e-6
        got = hr[f, y * B:(y + 1) * B, x * B:(x + 1) * B].astype(np.float64)
        assert np.abs(got - np.floor(e * 255.0 + 0.5)).max() <= 1
    assert n_rot > 0
    # with nothing turned the same call ignores the flag array
    hr0, _ = orc.unpack(frames, s, net, pl.places, place_rot=np.zeros(len(pl.places), dtype=np.int32))
    hr1, _ = orc.unpack(frames, s, net, pl.places)
    assert np.array_equal(hr0, hr1) and not np.array_equal(hr0, hr)


@pytest.mark.parametrize("topo", ["plain", "edsr"])
def test_exact_border_mode_equals_frame_based_everywhere(orc, topo):
    """Exact-border mode: with halo >= receptive-field radius the packed path equals plain
    frame-based SR of the frame at EVERY selected macroblock, border ones included (the plain
    mode only does so for interior ones); the whole-frame forward pass is the definition."""
    if topo == "plain":
        cfg, R = wl.config(1), 4                              # 4 convs
    else:
        cfg = wl.replace(wl.config(1), net=wl.Net("edsr", 6, 1, 2, 0.1), halo=6)
        R = 6                                                  # head, 2 block convs, body end, upsampler, tail(at x2: 1/2 px)
    frames, imp = wl.make_frames(cfg), wl.make_importance(cfg)
    imp[0, 0, :] += 5.0; imp[0, :, 0] += 5.0; imp[0, -1, -3:] += 5.0          # force border MBs into the selection
    blob = wl.make_weights(cfg.net, cfg.weight_seed, "fp32")
    segs = wl.make_segments(cfg)
    s, B = cfg.net.scale, 16 * cfg.net.scale
    full_plain = orc.sr_forward(cfg.net, blob, frames)[0]
    r = orc.run_path(frames, imp, segs, cfg.net, blob, cfg.halo, cfg.bin_size, exact_border=True)
    r0 = orc.run_path(frames, imp, segs, cfg.net, blob, cfg.halo, cfg.bin_size)
    n_border = n_fixed = 0
    for g, box, b, px, py in r.plan.places.tolist():
        y, x = divmod(g, cfg.mbw)
        want = full_plain[y * B:(y + 1) * B, x * B:(x + 1) * B]
        assert np.array_equal(r.net_out[b, py * s:py * s + B, px * s:px * s + B], want)
        if y in (0, cfg.mbh - 1) or x in (0, cfg.mbw - 1):
            n_border += 1
            n_fixed += not np.array_equal(r0.net_out[b, py * s:py * s + B, px * s:px * s + B], want)
    assert n_border >= 20 and n_fixed >= 10               # the plain mode really differs there
    # the mask itself: zero exactly on the out-of-frame part of the boxes
    keep = orc.border_keep(cfg.height, cfg.width, r.plan.boxes, cfg.halo, cfg.bin_size, r.plan.n_bins)
    zeros = 0
    for (f, x0, y0, w, h, rot, b, bx, by, bid) in r.plan.boxes.tolist():
        bw, bh = 16 * w + 2 * cfg.halo, 16 * h + 2 * cfg.halo
        ys = np.arange(16 * y0 - cfg.halo, 16 * y0 - cfg.halo + bh); xs = np.arange(16 * x0 - cfg.halo, 16 * x0 - cfg.halo + bw)
        inside = ((ys >= 0) & (ys < cfg.height))[:, None] & ((xs >= 0) & (xs < cfg.width))[None, :]
        assert np.array_equal(keep[b, by:by + bh, bx:bx + bw].astype(bool), inside)
        zeros += int((~inside).sum())
    assert int((keep == 0).sum()) == zeros > 0


def test_partial_macroblock_frames(orc):
    """Frame sides that are not multiples of 16: the macroblock grid is ceil(H/16) x ceil(W/16).
    (a) With every macroblock selected and the identity placement, the pasted frame is
    clamp(bilinear/255 + SR(frame)) over the whole true-size frame, computed here without any
    macroblock structure.  (b) The packed path zero-fills beyond the frame and pastes only the
    in-frame part of an edge macroblock; unselected macroblocks are the bilinear base."""
    cfg = wl.replace(wl.config(1), width=168, height=100, n_frames=2)
    assert (cfg.mbw, cfg.mbh) == (11, 7)
    frames, imp = wl.make_frames(cfg), wl.make_importance(cfg)
    assert frames.shape == (2, 100, 168, 3) and imp.shape == (2, 7, 11)
    blob = wl.make_weights(cfg.net, 0, "fp32")
    s = cfg.net.scale
    B = 16 * s
    # (a) frame-based
    net = orc.sr_forward(cfg.net, blob, frames)
    hr, sel = orc.unpack(frames, s, net, orc.identity_places(2, cfg.mbh, cfg.mbw))
    for f in range(2):
        base = orc.bilinear(frames[f], s).astype(np.float64) / 255.0
        e = np.clip(base + net[f], 0, 1)
        q = np.floor(e * 255.0 + 0.5)
        d = np.abs(hr[f].astype(np.float64) - q)
        assert hr[f].shape == (200, 336, 3) and d.max() <= 1 and (d > 0).mean() < 1e-3
    # the block of the bottom-right macroblock: in-frame part reported, the rest zero
    last = sel[cfg.mbw * cfg.mbh - 1]
    assert np.abs(last[:8, :16] - np.clip(orc.bilinear(frames[0], s)[192:, 320:].astype(np.float64) / 255.0 + net[0][192:, 320:], 0, 1)).max() < 1e-6
    assert not last[8:].any() and not last[:, 16:].any()
    # (b) packed path with edge macroblocks forced into the selection
    imp[:, -1, :] += 5.0; imp[:, :, -1] += 5.0
    r = orc.run_path(frames, imp, np.array([[0, 2, 60]], dtype=np.uint32), cfg.net, blob, cfg.halo, cfg.bin_size)
    assert r.mask[:, -1, :].all() and r.mask[:, :, -1].all()
    for (g, box, b, px, py), blk in zip(r.plan.places.tolist(), r.sel):
        f, rem = divmod(g, cfg.mbw * cfg.mbh); y, x = divmod(rem, cfg.mbw)
        h_in, w_in = min(16, 100 - 16 * y), min(16, 168 - 16 * x)
        want = np.zeros((16, 16, 3), dtype=np.uint8); want[:h_in, :w_in] = frames[f, 16 * y:16 * y + h_in, 16 * x:16 * x + w_in]
        assert np.array_equal(r.bins[b, py:py + 16, px:px + 16], want)          # zero beyond the frame
        base = orc.bilinear(frames[f], s)[y * B:y * B + h_in * s, x * B:x * B + w_in * s].astype(np.float64) / 255.0
        e = np.clip(base + r.net_out[b, py * s:py * s + h_in * s, px * s:px * s + w_in * s], 0, 1)
        assert np.abs(blk[:h_in * s, :w_in * s] - e).max() < 1e-6
        assert not blk[h_in * s:].any() and not blk[:, w_in * s:].any()
    for f in range(2):
        base = orc.bilinear(frames[f], s)
        keep = ~np.kron(r.mask[f], np.ones((B, B), dtype=np.uint8)).astype(bool)[:200, :336]
        assert np.array_equal(r.frames_hr[f][keep], base[keep])


def test_place_that_leaves_the_enhanced_image_stays_bilinear(orc):
    """A place is honoured only when the in-frame part of its macroblock lies inside the enhanced
    image; otherwise the macroblock keeps the bilinear base and sel reports zeros.  Hand case: one
    4 x 3 macroblock frame, an enhanced image of 40 x 24 low-resolution pixels, four places."""
    rng = np.random.default_rng(5)
    s, B = 2, 32
    frame = rng.integers(0, 256, size=(1, 48, 64, 3), dtype=np.uint8)
    net = rng.normal(0.0, 0.1, size=(1, 24 * s, 40 * s, 3))
    base = orc.bilinear(frame[0], s)
    #          mb_id box bin  px  py
    places = [[0, 0, 0, 0, 0],        # inside: pasted
              [1, 0, 0, 24, 8],       # px + 16 = 40 <= 40, py + 16 = 24 <= 24: just inside, pasted
              [5, 0, 0, 25, 0],       # px + 16 = 41 > 40: leaves the image on the right
              [6, 0, 0, 0, 9],        # py + 16 = 25 > 24: leaves it at the bottom
              [7, 0, 0xFFFF, 0, 0]]   # not placed at all
    hr, sel = orc.unpack(frame, s, net, np.array(places, dtype=np.int32))
    for i, (g, _, b, px, py) in enumerate(places):
        y, x = divmod(g, 4)
        got = hr[0, y * B:(y + 1) * B, x * B:(x + 1) * B]
        bb = base[y * B:(y + 1) * B, x * B:(x + 1) * B]
        if i < 2:
            e = np.clip(bb.astype(np.float64) / 255.0 + net[0, py * s:py * s + B, px * s:px * s + B], 0, 1)
            assert np.abs(sel[i] - e).max() < 1e-6 and (got != bb).any()
            assert np.abs(got.astype(np.float64) - np.floor(e * 255.0 + 0.5)).max() <= 1
        else:
            assert np.array_equal(got, bb) and not sel[i].any()
    # every macroblock without a place is the base as well
    untouched = np.ones((3, 4), dtype=bool); untouched[0, 0] = untouched[0, 1] = False
    keep = np.kron(untouched, np.ones((B, B), dtype=bool))
    assert np.array_equal(hr[0][keep], base[keep])
    # a turned place swaps the roles of the two extents: 16 x 16 blocks are symmetric, a cut block is not
    frame2 = rng.integers(0, 256, size=(1, 40, 64, 3), dtype=np.uint8)         # bottom macroblock row is 8 pixels tall
    net2 = rng.normal(0.0, 0.1, size=(1, 24 * s, 40 * s, 3))
    pl = np.array([[8, 0, 0, 30, 0], [9, 0, 0, 30, 0]], dtype=np.int32)        # both in the cut row (y = 2)
    # upright needs 16 columns x 8 rows: 30 + 16 > 40 -> leaves; turned needs 8 columns x 16 rows: 30 + 8 <= 40 -> pasted
    hr2, sel2 = orc.unpack(frame2, s, net2, pl, place_rot=np.array([0, 1], dtype=np.int32))
    base2 = orc.bilinear(frame2[0], s)
    assert np.array_equal(hr2[0, 64:80, 0:32], base2[64:80, 0:32]) and not sel2[0].any()
    e = np.clip(base2[64:80, 32:64].astype(np.float64) / 255.0 + net2[0, 0:32, 60:76].transpose(1, 0, 2), 0, 1)
    assert np.abs(sel2[1][:16] - e).max() < 1e-6 and not sel2[1][16:].any()
