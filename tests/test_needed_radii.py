"""The needed-region mode's layer radii (rh_needed_radii, host logic of the library).

Claim: if every layer's output is right only within its radius (Chebyshev distance, in
low-resolution pixels) of the pasted pixels, the network output on the pasted pixels is still the
plain forward's, bit for bit.  Checked with the network composed from library convs in fp64 and
NaN written everywhere outside a layer's radius: a single read across the boundary would poison
the result.  The schedule is also tight: with every radius one smaller the poison arrives."""
import numpy as np
import pytest
import torch
import torch.nn.functional as TF
from scipy.ndimage import binary_dilation

import workloads as wl
from paper_2407_16990_amd import needed_radii

NETS = [wl.Net("edsr", 4, 2, 2), wl.Net("edsr", 4, 1, 4), wl.Net("edsr", 4, 3, 3), wl.Net("res", 4, 2, 2), wl.Net("res", 4, 1, 3),
        wl.Net("plain", 4, 4, 2), wl.Net("plain", 4, 2, 2)]


def dilate(M, r):
    return M if r == 0 else binary_dilation(M, structure=np.ones((3, 3), dtype=bool), iterations=r)


def forward(net, blob, img, M=None, radii=None):
    """Library composition; with M and radii, every layer's output is NaN outside its radius."""
    layers, pos = [], 0
    for cin, cout, _ in wl.net_layers(net):
        w = torch.from_numpy(blob[pos:pos + cout * 9 * cin].reshape(cout, 3, 3, cin)).permute(0, 3, 1, 2).double(); pos += cout * 9 * cin
        b = torch.from_numpy(blob[pos:pos + cout]).double(); pos += cout
        layers.append((w, b))
    it = iter(layers)
    conv = lambda t: TF.conv2d(t, *next(it), padding=1)
    k = [0]

    def cut(t):                                               # layer k's output, valid within its radius only
        if M is not None:
            keep = torch.from_numpy(dilate(M, radii[k[0]]))[None, None]
            t = torch.where(keep, t, torch.full_like(t, float("nan")))
        k[0] += 1
        return t
    x = torch.from_numpy(img.astype(np.float64) / 255.0).permute(2, 0, 1)[None]
    if net.topology == "plain":
        x = cut(torch.relu(conv(x)))
        for _ in range(net.n_blocks - 2):
            x = cut(torch.relu(conv(x)))
        y = TF.pixel_shuffle(conv(x), net.scale)
    else:
        x = cut(conv(x)); head = x
        for _ in range(net.n_blocks):
            t = cut(torch.relu(conv(x)))
            x = cut(x + conv(t))
        if net.topology == "res":
            y = TF.pixel_shuffle(conv(x), net.scale)
        else:
            x = cut(conv(x) + head)
            for _ in range(2 if net.scale == 4 else 1):
                x = TF.pixel_shuffle(conv(x), 2 if net.scale == 4 else net.scale)
            y = conv(x)
    if radii is not None:
        assert k[0] == len(radii) - 1 and radii[-1] == 0
    return y[0].permute(1, 2, 0).numpy()


def pasted_mask(rng, H, W, n=3):
    M = np.zeros((H, W), dtype=bool)
    for _ in range(n):
        y, x = int(rng.integers(0, H - 16 + 1)), int(rng.integers(0, W - 16 + 1))
        M[y:y + 16, x:x + 16] = True
    return M


@pytest.mark.parametrize("net", NETS, ids=lambda n: f"{n.topology}{n.n_blocks}x{n.scale}")
def test_layers_right_within_their_radius_give_the_plain_output_on_the_pasted_pixels(net):
    radii = needed_radii(net)
    nb = {"edsr": 2 * net.n_blocks + 1, "res": 2 * net.n_blocks, "plain": net.n_blocks - 2}[net.topology]
    assert radii is not None and len(radii) == nb + 2 and radii[-1] == 0
    assert all(a == b + 1 for a, b in zip(radii[:-2], radii[1:-1]))          # one pixel of reach per conv
    rng = np.random.default_rng(21)
    blob = wl.make_weights(net, 9, "fp32")
    H, W, s = 72, 104, net.scale
    tight = 0
    for trial in range(3):
        img = rng.integers(0, 256, size=(H, W, 3), dtype=np.uint8)
        M = pasted_mask(rng, H, W)
        Mhr = np.kron(M, np.ones((s, s), dtype=bool))
        plain = forward(net, blob, img)
        cutout = forward(net, blob, img, M, radii)
        assert not np.isnan(cutout[Mhr]).any()
        assert np.array_equal(cutout[Mhr], plain[Mhr])
        assert np.isnan(cutout[~Mhr]).any()                                   # the rest really was cut away
        short = forward(net, blob, img, M, [max(r - 1, 0) for r in radii[:-1]] + [0])
        tight += int(np.isnan(short[Mhr]).any())
    assert tight == 3                                                          # one pixel less anywhere is too little


def test_networks_the_mode_does_not_cover():
    assert needed_radii(wl.Net("edsr", 64, 2, 4), per_layer_tail=True) is None
    assert needed_radii(wl.Net("edsr", 64, 300, 4)) is None                    # more layers than the table holds
