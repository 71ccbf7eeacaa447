"""Pins of the oracle's box-masked enhance mode (Sec. 3.3.2: bins are only partly occupied).

The mode zeroes the first conv's and every body conv's output outside the cells that a placed
box touches and runs the layers after the body unmasked.  The pins: the cell map against a
hand-drawn case; the masked forward against the same network composed from library ops with the
mask multiplied in; keep = 1 everywhere reproduces the plain forward bit for bit; keep = 0
everywhere leaves the closed form "tail of a zero tensor"; and with one live cell the output far
from it is that closed form while the cell's interior equals the plain forward."""
import numpy as np
import pytest
import torch
import torch.nn.functional as TF

import workloads as wl

NETS = [wl.Net("plain", 8, 4, 2), wl.Net("res", 8, 2, 3), wl.Net("edsr", 8, 2, 2), wl.Net("edsr", 6, 2, 3),
        wl.Net("edsr", 8, 1, 4)]


def layers_of(net, blob):
    pos, out = 0, []
    for cin, cout, _ in wl.net_layers(net):
        w = torch.from_numpy(blob[pos:pos + cout * 9 * cin].reshape(cout, 3, 3, cin)).permute(0, 3, 1, 2).double(); pos += cout * 9 * cin
        b = torch.from_numpy(blob[pos:pos + cout]).double(); pos += cout
        out.append((w, b))
    assert pos == len(blob)
    return out


def t_net_masked(net, blob, img, keep):
    """Library composition with the mask applied after the first conv and every body conv."""
    x = torch.from_numpy(img.astype(np.float64) / 255.0).permute(2, 0, 1)[None]
    m = torch.from_numpy(keep.astype(np.float64))[None, None]
    it = iter(layers_of(net, blob))
    conv = lambda t: TF.conv2d(t, *next(it), padding=1)
    if net.topology == "plain":
        for _ in range(net.n_blocks - 1):
            x = torch.relu(conv(x)) * m
        y = TF.pixel_shuffle(conv(x), net.scale)
    else:
        x = conv(x) * m; head = x
        for _ in range(net.n_blocks):
            x = (x + conv(torch.relu(conv(x)) * m)) * m
        if net.topology == "res":
            y = TF.pixel_shuffle(conv(x), net.scale)
        else:
            x = (conv(x) + head) * m
            for _ in range(2 if net.scale == 4 else 1):
                x = TF.pixel_shuffle(conv(x), 2 if net.scale == 4 else net.scale)
            y = conv(x)
    return y[0].permute(1, 2, 0).numpy()


def test_cell_keep_hand_case(orc):
    """Rows: frame, mbx0, mby0, wmb, hmb, rot, bin, bx, by, id.  halo 3, 64 x 64 bins, 16 x 32 cells."""
    boxes = np.array([
        [0, 0, 0, 1, 1, 0, 0, 0, 0, 0],        # 22 x 22 at (0, 0): rows 0..21 -> cell rows 0, 1; cols 0..21 -> cell col 0
        [0, 5, 5, 2, 1, 1, 1, 40, 20, 1],      # 38 x 22 turned -> 22 wide, 38 tall at (40, 20): cols 40..61, rows 20..57
        [0, 9, 9, 1, 1, 0, 2, 31, 15, 2],      # 22 x 22 at (31, 15): cols 31..52 -> both cell cols; rows 15..36 -> cell rows 0..2
        [0, 3, 3, 1, 1, 0, 0xFFFF, 0, 0, 3],   # did not fit: no bin
    ], dtype=np.int32)
    keep = orc.cell_keep(boxes, 3, 64, 4, cell_h=16, cell_w=32)
    want = np.zeros((4, 64, 64), dtype=np.uint8)
    want[0, 0:32, 0:32] = 1
    want[1, 16:64, 32:64] = 1
    want[2, 0:48, 0:64] = 1
    assert np.array_equal(keep, want)
    # a bin whose side is not a multiple of the cell: the cut cells at the edge
    keep = orc.cell_keep(np.array([[0, 0, 0, 1, 1, 0, 0, 26, 26, 0]], dtype=np.int32), 3, 48, 1, cell_h=16, cell_w=32)
    want = np.zeros((1, 48, 48), dtype=np.uint8)
    want[0, 16:48, 0:48] = 1                    # rows 26..47 -> cell rows 1, 2; cols 26..47 -> cell cols 0 and the cut cell 1
    assert np.array_equal(keep, want)
    # the library's cells (the default): 8 rows x 32 columns
    keep = orc.cell_keep(boxes, 3, 64, 4)
    want = np.zeros((4, 64, 64), dtype=np.uint8)
    want[0, 0:24, 0:32] = 1                     # rows 0..21 -> rows of 8: 0, 1, 2
    want[1, 16:64, 32:64] = 1                   # rows 20..57 -> 2..7
    want[2, 8:40, 0:64] = 1                     # rows 15..36 -> 1..4
    assert np.array_equal(keep, want)


@pytest.mark.parametrize("net", NETS)
def test_masked_forward_vs_library_composition(orc, net):
    rng = np.random.default_rng(11)
    blob = wl.make_weights(net, 4, "fp32")
    imgs = rng.integers(0, 256, size=(2, 12, 16, 3), dtype=np.uint8)
    keep = np.kron(rng.integers(0, 2, size=(2, 3, 2), dtype=np.uint8), np.ones((4, 8), dtype=np.uint8))
    assert 0 < keep.sum() < keep.size
    out = orc.sr_forward(net, blob, imgs, keep, body_only=True)
    for n in range(2):
        want = t_net_masked(net, blob, imgs[n], keep[n])
        assert np.allclose(out[n], want, rtol=1e-11, atol=1e-11)
    # it is a different function from the plain forward and from the all-layer mask
    assert not np.allclose(out, orc.sr_forward(net, blob, imgs), atol=1e-6)
    if net.topology == "edsr":
        assert not np.allclose(out, orc.sr_forward(net, blob, imgs, keep), atol=1e-6)


@pytest.mark.parametrize("net", NETS)
def test_masked_forward_with_everything_kept_is_the_plain_forward(orc, net):
    rng = np.random.default_rng(12)
    blob = wl.make_weights(net, 5, "fp32")
    imgs = rng.integers(0, 256, size=(1, 10, 9, 3), dtype=np.uint8)
    assert np.array_equal(orc.sr_forward(net, blob, imgs, np.ones((1, 10, 9), dtype=np.uint8), body_only=True),
                          orc.sr_forward(net, blob, imgs))


def tail_of_zero(net, blob, y, x):
    """Closed form of the network output at interior pixel (y, x) when the body's output is zero."""
    L = layers_of(net, blob)
    s = net.scale
    if net.topology != "edsr":
        b = L[-1][1].numpy()                                   # conv of zeros = bias, then the shuffle
        return np.array([b[c * s * s + (y % s) * s + (x % s)] for c in range(3)])
    assert s in (2, 3)
    bu = L[-2][1].numpy(); wl_, bl = L[-1][0].numpy(), L[-1][1].numpy()      # wl_[co][ci][ky][kx]
    C = net.channels
    P = lambda yy, xx, ci: bu[ci * s * s + (yy % s) * s + (xx % s)]         # the shuffled upsampler bias
    return np.array([bl[c] + sum(wl_[c, ci, ky, kx] * P(y + ky - 1, x + kx - 1, ci)
                                 for ci in range(C) for ky in range(3) for kx in range(3)) for c in range(3)])


@pytest.mark.parametrize("net", [wl.Net("plain", 8, 3, 2), wl.Net("res", 8, 2, 3), wl.Net("edsr", 8, 2, 2), wl.Net("edsr", 6, 1, 3)])
def test_nothing_kept_leaves_the_tail_of_a_zero_tensor(orc, net):
    rng = np.random.default_rng(13)
    blob = wl.make_weights(net, 6, "fp32")
    imgs = rng.integers(0, 256, size=(1, 8, 8, 3), dtype=np.uint8)
    out = orc.sr_forward(net, blob, imgs, np.zeros((1, 8, 8), dtype=np.uint8), body_only=True)[0]
    s = net.scale
    for (y, x) in [(1, 1), (2, 5), (s * 4 + 1, s * 3 + 2), (8 * s - 2, 8 * s - 2)]:
        assert np.allclose(out[y, x], tail_of_zero(net, blob, y, x), rtol=1e-12, atol=1e-13)
    assert np.abs(out).max() > 0                               # the biases are not zero: the tail is not masked


def test_one_live_cell_far_field_and_interior(orc):
    """3 x 3 cells of 16 x 32 pixels, only the centre one kept.  EDSR, 1 block, x2: the tail reaches
    2 low-resolution pixels, the whole net 6.  Farther than 2 pixels from the cell the output is the
    tail of zero (a mask missing after the residual or long-skip addition would leak the first
    conv's output there); deeper than 6 pixels inside the cell it equals the plain forward."""
    net = wl.Net("edsr", 6, 1, 2)
    rng = np.random.default_rng(14)
    blob = wl.make_weights(net, 7, "fp32")
    img = rng.integers(0, 256, size=(1, 48, 96, 3), dtype=np.uint8)
    keep = np.zeros((1, 48, 96), dtype=np.uint8); keep[0, 16:32, 32:64] = 1
    out = orc.sr_forward(net, blob, img, keep, body_only=True)[0]
    zero = orc.sr_forward(net, blob, img, np.zeros_like(keep), body_only=True)[0]
    plain = orc.sr_forward(net, blob, img)[0]
    far = np.ones((96, 192), dtype=bool); far[2 * (16 - 2):2 * (32 + 2), 2 * (32 - 2):2 * (64 + 2)] = False
    assert np.array_equal(out[far], zero[far])
    near = ~far
    assert not np.array_equal(out[near], zero[near])
    inner = (slice(2 * (16 + 6), 2 * (32 - 6)), slice(2 * (32 + 6), 2 * (64 - 6)))
    assert np.array_equal(out[inner], plain[inner])
    edge = (slice(2 * 16, 2 * 18), slice(2 * 32, 2 * 64))      # just inside the cell: the zeros outside are felt
    assert not np.array_equal(out[edge], plain[edge])


def test_run_path_box_masked_pastes_the_masked_output(orc):
    cfg = wl.config(1)
    frames, imp, segs = wl.make_frames(cfg), wl.make_importance(cfg), wl.make_segments(cfg)
    blob = wl.make_weights(cfg.net, cfg.weight_seed, "fp32")
    r = orc.run_path(frames, imp, segs, cfg.net, blob, cfg.halo, cfg.bin_size, box_masked=True)
    keep = orc.cell_keep(r.plan.boxes, cfg.halo, cfg.bin_size, r.plan.n_bins)
    assert 0 < keep.mean() < 1
    assert np.array_equal(r.net_out, orc.sr_forward(cfg.net, blob, r.bins, keep, body_only=True))
    s = cfg.net.scale
    for i, (g, box, b, px, py) in enumerate(r.plan.places.tolist()):       # every placed macroblock lies in kept cells
        assert keep[b, py:py + 16, px:px + 16].all()
    assert r.sel.shape[0] == len(r.plan.places)
