"""GPU parity of the temporal importance reuse step (Sec. 3.2.2) against the CPU oracle, through
the C ABI.  Everything here is integer or a copy: the bar is bit-exact."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import temporal as OT
from paper_2407_16990_amd import RH

pytestmark = pytest.mark.gpu

NET = wl.Net("plain", 4, 2, 2)


def make_ctx(w, h, max_frames):
    return RH(frame_w=w, frame_h=h, max_frames=max_frames, halo=2, bin_size=32, max_bins=4, net=NET,
              weights=wl.make_weights(NET, 0, "fp32"), precision="fp32")


def gpu_phi(rh, res, tau, min_area):
    out = rh.temporal_phi(torch.from_numpy(res).cuda(), tau, min_area)
    return out.cpu().numpy().view(np.uint64)


def check_phi(res, tau, min_area, rh=None):
    own = rh is None
    if own:
        rh = make_ctx(res.shape[2], res.shape[1], res.shape[0])
    want, _ = OT.phi(res, tau, min_area)
    got = gpu_phi(rh, res, tau, min_area)
    assert np.array_equal(got, want), (got, want)
    if own:
        rh.close()
    return want


@pytest.mark.parametrize("w,h,streams,fps", [(480, 272, 2, 8), (640, 368, 8, 4)])
def test_phi_on_synthetic_residuals_at_full_size(w, h, streams, fps):
    res = wl.make_residuals(w, h, streams, fps, seed=w)
    rh = make_ctx(w, h, streams * fps)
    for tau, min_area in [(12, 1), (12, 4), (6, 2), (40, 1)]:
        print(f"[phi {w}x{h} F={streams * fps}] tau={tau} min_area={min_area}", flush=True)
        check_phi(res, tau, min_area, rh)
    # a second call with fewer frames on the same context (workspace reuse)
    check_phi(res[:3], 12, 1, rh)
    rh.close()


@pytest.mark.parametrize("density", [0.0, 0.02, 0.2, 0.45, 0.6, 0.9, 1.0])
@pytest.mark.parametrize("w,h", [(16, 16), (19, 17), (53, 37), (64, 16), (130, 67), (257, 33)])
def test_phi_random_masks_ragged_sizes(density, w, h):
    rng = np.random.default_rng(int(density * 100) + w)
    res = ((rng.random((5, h, w)) < density) * rng.integers(20, 200, (5, h, w))).astype(np.int16)
    res *= rng.choice(np.array([-1, 1], dtype=np.int16), size=res.shape)
    check_phi(res, 10, 1)
    check_phi(res, 10, 3)


def test_phi_shapes_that_stress_the_labelling():
    H, W = 70, 200
    imgs = []
    snake = np.zeros((H, W), dtype=np.int16)                      # one-pixel serpentine across segment borders
    for y in range(0, H, 2):
        snake[y, :] = 40
        if y + 1 < H:
            snake[y + 1, W - 1 if (y // 2) % 2 == 0 else 0] = 40
    imgs.append(snake)
    vsnake = np.zeros((H, W), dtype=np.int16)                     # the same, turned
    for x in range(0, W, 2):
        vsnake[:, x] = -40
        if x + 1 < W:
            vsnake[H - 1 if (x // 2) % 2 == 0 else 0, x + 1] = -40
    imgs.append(vsnake)
    diag = np.zeros((H, W), dtype=np.int16)                       # diagonals both ways: 8-neighbour contacts only
    for i in range(min(H, W)):
        diag[i, i] = 99
        diag[i, W - 1 - i] = 99
    imgs.append(diag)
    checker = np.zeros((H, W), dtype=np.int16); checker[::2, ::2] = 30; checker[1::2, 1::2] = 30   # one blob by diagonals
    imgs.append(checker)
    dots = np.zeros((H, W), dtype=np.int16); dots[::2, ::2] = 30  # the most blobs a frame can hold
    imgs.append(dots)
    full = np.full((H, W), 77, dtype=np.int16)
    imgs.append(full)
    rings = np.zeros((H, W), dtype=np.int16)                      # nested rings: separate blobs
    for k in range(0, 30, 4):
        rings[k:H - k, k] = 50; rings[k:H - k, W - 1 - k] = 50; rings[k, k:W - k] = 50; rings[H - 1 - k, k:W - k] = 50
    imgs.append(rings)
    comb = np.zeros((H, W), dtype=np.int16); comb[0, :] = 60; comb[:, ::3] = 60    # many columns joined by one row
    imgs.append(comb)
    res = np.stack(imgs)
    want = check_phi(res, 10, 1)
    assert int(want[0]) == (1 << 32) // int((snake != 0).sum())
    assert int(want[4]) == (H // 2) * (W // 2) * (1 << 32)
    check_phi(res, 10, 5)


def run_select(rh, phi_q, off, n_total):
    d_phi = torch.from_numpy(phi_q.view(np.int64)).cuda()
    alloc, sel, reuse, n_sel = rh.temporal_select(d_phi, off, n_total)
    o_alloc, o_sel, o_reuse = OT.temporal_plan(phi_q, off, n_total)
    assert alloc.cpu().numpy().tolist() == o_alloc
    assert np.array_equal(sel.cpu().numpy(), o_sel)
    assert np.array_equal(reuse.cpu().numpy().astype(np.uint32), o_reuse)
    assert int(n_sel.cpu()[0]) == int(o_sel.sum())
    return sel, reuse


@pytest.mark.parametrize("seed", range(6))
def test_select_random_streams(seed):
    rng = np.random.default_rng(seed)
    ns = int(rng.integers(1, 12))
    lens = rng.integers(1, 70, ns)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    F = int(off[-1])
    rh = make_ctx(64, 48, F)
    phi_q = rng.integers(0, 1 << 40, F).astype(np.uint64)
    if seed % 2:                                                  # plateaus and still streams
        phi_q = phi_q[np.arange(F) - np.arange(F) % 4]
        b, e = off[0], off[1]
        phi_q[b:e] = phi_q[b]
    for n_total in (ns, ns + 1, ns + 7, 3 * F):
        print(f"[select seed={seed}] streams={ns} F={F} budget={n_total}", flush=True)
        run_select(rh, phi_q, off, n_total)
    rh.close()


def test_select_from_the_operator_and_spread():
    w, h, streams, fps = 160, 96, 4, 12
    res = wl.make_residuals(w, h, streams, fps, seed=5)
    F = streams * fps
    rh = make_ctx(w, h, F)
    d_phi = rh.temporal_phi(torch.from_numpy(res).cuda(), 12, 2)
    phi_q = d_phi.cpu().numpy().view(np.uint64)
    assert np.array_equal(phi_q, OT.phi(res, 12, 2)[0])
    off = [fps * s for s in range(streams + 1)]
    sel, reuse = run_select(rh, phi_q, off, 14)
    rng = np.random.default_rng(9)
    imp = rng.random((F, rh.mbh, rh.mbw)).astype(np.float32)
    want = OT.spread(imp, reuse.cpu().numpy())
    got = rh.temporal_spread(torch.from_numpy(imp).cuda(), sel, reuse).cpu().numpy()
    assert np.array_equal(got, want)
    rh.close()


def test_select_extremes():
    rh = make_ctx(16, 16, 4096)
    rng = np.random.default_rng(3)
    # the longest chunk, values near the largest Phi such a frame can give
    phi_q = rng.integers(0, 81 << 32, 2048).astype(np.uint64)
    run_select(rh, phi_q, [0, 2048], 300)
    run_select(rh, phi_q, [0, 2048], 65535)
    # nothing changes anywhere: equal shares, first frames
    flat = np.full(40, 5 << 32, dtype=np.uint64)
    run_select(rh, flat, [0, 10, 20, 40], 9)
    # 1024 one- and two-frame streams
    off = np.concatenate([[0], np.cumsum(rng.integers(1, 3, 1024))])
    phi_q = rng.integers(0, 1 << 36, int(off[-1])).astype(np.uint64)
    run_select(rh, phi_q, off, 1500)
    rh.close()


def test_temporal_argument_errors():
    rh = make_ctx(64, 48, 8)
    res = torch.zeros((8, 48, 64), dtype=torch.int16, device="cuda")
    phi = rh.temporal_phi(res, 5, 1)
    assert phi.cpu().numpy().tolist() == [0] * 8
    with pytest.raises(RuntimeError):
        rh.temporal_phi(res, -1, 1)
    with pytest.raises(RuntimeError):
        rh.temporal_phi(res, 5, 0)
    with pytest.raises(RuntimeError):
        rh.temporal_phi(torch.zeros((9, 48, 64), dtype=torch.int16, device="cuda"), 5, 1)      # more than max_frames
    with pytest.raises(RuntimeError):
        rh.temporal_select(phi, [0, 8], 0)                        # budget below one frame per stream
    with pytest.raises(RuntimeError):
        rh.temporal_select(phi, [0, 4, 4, 8], 5)                  # an empty stream
    with pytest.raises(RuntimeError):
        rh.temporal_select(phi, [1, 8], 5)                        # does not start at frame 0
    alloc, sel, reuse, n = rh.temporal_select(phi, [0, 8], 3)     # and a valid call still works afterwards
    assert sel.cpu().numpy().tolist() == [1, 0, 0, 0, 0, 0, 0, 0] and int(n.cpu()[0]) == 1
    rh.close()
