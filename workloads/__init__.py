"""Seeded synthetic workloads for the region-aware enhancer.

This module only *draws inputs*: frames, macroblock importance maps, selection
segments and network weights, in the shapes of the five benchmark
configurations.  It contains none of the method's arithmetic (no selection,
packing, convolution, interpolation) and is the one module both the CPU oracle
tests and the HIP path's tests/bench import, so both sides see identical bytes.

The inputs stand in for the paper's video datasets (360p-class streams,
16x16 macroblocks, 10-25 % of the frame area worth enhancing, clustered in a
few regions; Sec. 2.3 and Sec. 4.1), which are not available here.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np

MB = 16  # macroblock side in input pixels (H.264; Sec. 3.2.1)


@dataclass(frozen=True)
class Net:
    """SR network descriptor.  topology: 'plain' | 'res' | 'edsr'."""
    topology: str
    channels: int
    n_blocks: int   # plain: total number of conv layers; res/edsr: residual blocks
    scale: int
    tail_scale: float = 0.1   # multiplier on the last conv's He-normal weights


@dataclass(frozen=True)
class Config:
    name: str
    index: int
    n_frames: int
    width: int
    height: int
    halo: int
    bin_size: int
    net: Net
    precision: str               # 'fp32' | 'bf16'
    weight_seed: int
    n_streams: int = 1           # frames are split evenly over streams, in order
    frac: float = 0.2            # selected fraction (per stream: drawn if frac_range set)
    frac_range: Tuple[float, float] | None = None
    blobs: Tuple[int, int] = (3, 3)   # inclusive range of importance blobs per frame
    lognormal_amp: bool = False
    importance: str = "clustered"     # 'clustered' | 'uniform'
    quantize_levels: int = 0          # >0: importance quantised to that many levels (tie stress)

    @property
    def mbw(self) -> int:
        return (self.width + MB - 1) // MB      # a partial macroblock at the right edge counts

    @property
    def mbh(self) -> int:
        return (self.height + MB - 1) // MB

    @property
    def n_mbs(self) -> int:
        return self.n_frames * self.mbw * self.mbh


# last-conv scale of the benchmark nets: network output of rms about 0.05 (a correction to the
# interpolated frame of a few hundredths of the pixel range, as a trained SR net's is)
EDSR_X4 = Net("edsr", 64, 16, 4, tail_scale=0.0125)
EDSR_X3 = Net("edsr", 64, 16, 3, tail_scale=0.0125)

CONFIGS: List[Config] = [
    Config("cfg1_320x192_plain16_x2_fp32", 1, 1, 320, 192, 4, 64,
           Net("plain", 16, 4, 2, tail_scale=0.1), "fp32", 0, frac=0.25, blobs=(2, 2)),
    Config("cfg2_8x640x368_res32_x2_bf16", 2, 8, 640, 368, 6, 96,
           Net("res", 32, 8, 2, tail_scale=0.03), "bf16", 0, frac=0.30, blobs=(1, 4)),
    Config("cfg3_16x480x272_edsr64_x4_bf16", 3, 16, 480, 272, 10, 128,
           EDSR_X4, "bf16", 1, frac=0.20, blobs=(3, 3)),
    # cfg4 = cfg3 with the fraction swept; see with_frac() / with_importance()
    Config("cfg4_sweep_edsr64_x4_bf16", 4, 16, 480, 272, 10, 128,
           EDSR_X4, "bf16", 1, frac=0.20, blobs=(3, 3)),
    Config("cfg5_8streams_x4_640x368_edsr64_x3_bf16", 5, 32, 640, 368, 10, 128,
           EDSR_X3, "bf16", 1, n_streams=8, frac_range=(0.05, 0.5), blobs=(1, 4),
           lognormal_amp=True),
]


def config(i: int) -> Config:
    """Configuration by its 1-based number (the order of the benchmark list)."""
    return CONFIGS[i - 1]


def replace(cfg: Config, **kw) -> Config:
    import dataclasses
    return dataclasses.replace(cfg, **kw)


# ---------------------------------------------------------------------------
# network layer table (blob format only: which convs, in which order)
# ---------------------------------------------------------------------------

def net_layers(net: Net) -> List[Tuple[int, int, str]]:
    """(cin, cout, role) of every 3x3 conv in weight-blob order.

    role in {'relu', 'linear', 'res2', 'last'} drives only the init scaling
    below; the meaning of each layer is defined by the C header.
    """
    C, s = net.channels, net.scale
    L: List[Tuple[int, int, str]] = []
    if net.topology == "plain":
        assert net.n_blocks >= 2
        L.append((3, C, "relu"))
        for _ in range(net.n_blocks - 2):
            L.append((C, C, "relu"))
        L.append((C, 3 * s * s, "last"))
    elif net.topology == "res":
        L.append((3, C, "linear"))
        for _ in range(net.n_blocks):
            L.append((C, C, "relu"))
            L.append((C, C, "res2"))
        L.append((C, 3 * s * s, "last"))
    elif net.topology == "edsr":
        L.append((3, C, "linear"))
        for _ in range(net.n_blocks):
            L.append((C, C, "relu"))
            L.append((C, C, "res2"))
        L.append((C, C, "linear"))
        if s in (2, 3):
            L.append((C, C * s * s, "linear"))
        elif s == 4:
            L.append((C, 4 * C, "linear"))
            L.append((C, 4 * C, "linear"))
        else:
            raise ValueError("edsr scale must be 2, 3 or 4")
        L.append((C, 3, "last"))
    else:
        raise ValueError(net.topology)
    return L


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even), returned as float32."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = (u + 0x7FFF + lsb) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(x.shape)


def make_weights(net: Net, seed: int, precision: str) -> np.ndarray:
    """Flat float32 blob: per layer w[cout][ky][kx][cin] then b[cout].

    He-normal weights (std = sqrt(2 / (9 cin))); the second conv of every
    residual block is scaled by 1/sqrt(n_blocks) and the last conv by
    net.tail_scale so that the network's output is a small correction to the
    interpolated frame; biases are small and non-zero so that a dropped bias is
    visible.  For 'bf16' every value is rounded once, here, to a bf16-exact
    float32.
    """
    rng = np.random.Generator(np.random.PCG64(1_000_003 * (seed + 1)))
    parts = []
    for cin, cout, role in net_layers(net):
        w = rng.standard_normal((cout, 3, 3, cin)).astype(np.float32)
        w *= np.float32(np.sqrt(2.0 / (9.0 * cin)))
        b = (rng.uniform(-0.05, 0.05, size=cout)).astype(np.float32)
        if role == "res2":
            w *= np.float32(1.0 / np.sqrt(net.n_blocks))
        elif role == "last":
            w *= np.float32(net.tail_scale)
            b *= np.float32(net.tail_scale)
        parts += [w.ravel(), b]
    blob = np.concatenate(parts).astype(np.float32)
    if precision == "bf16":
        blob = round_to_bf16(blob)
    return blob


# ---------------------------------------------------------------------------
# frames, importance maps, segments
# ---------------------------------------------------------------------------

def make_frames(cfg: Config, n_frames: int | None = None) -> np.ndarray:
    """uint8 [F, H, W, 3]: half uniform noise, half three smooth Gaussian blobs."""
    F = cfg.n_frames if n_frames is None else n_frames
    H, W = cfg.height, cfg.width
    out = np.empty((F, H, W, 3), dtype=np.uint8)
    yy, xx = np.mgrid[0:H, 0:W].astype(np.float64)
    for f in range(F):
        rng = np.random.Generator(np.random.PCG64(cfg.index * 1000 + f))
        noise = rng.integers(0, 256, size=(H, W, 3)).astype(np.float64)
        smooth = np.zeros((H, W, 3), dtype=np.float64)
        for _ in range(3):
            cx, cy = rng.uniform(0, W), rng.uniform(0, H)
            sig = rng.uniform(0.1, 0.3) * min(W, H)
            amp = rng.uniform(0.3, 1.0, size=3)
            g = np.exp(-((xx - cx) ** 2 + (yy - cy) ** 2) / (2 * sig * sig))
            smooth += g[:, :, None] * amp[None, None, :]
        img = 0.5 * noise + 0.5 * 255.0 * smooth
        out[f] = np.clip(np.rint(img), 0, 255).astype(np.uint8)
    return out


def make_importance(cfg: Config, n_frames: int | None = None) -> np.ndarray:
    """float32 [F, MBH, MBW] macroblock importance."""
    F = cfg.n_frames if n_frames is None else n_frames
    mbh, mbw = cfg.mbh, cfg.mbw
    rng = np.random.Generator(np.random.PCG64(77_000 + cfg.index * 1000))
    imp = np.empty((F, mbh, mbw), dtype=np.float64)
    yy, xx = np.mgrid[0:mbh, 0:mbw].astype(np.float64)
    for f in range(F):
        if cfg.importance == "uniform":
            imp[f] = rng.uniform(0.0, 1.0, size=(mbh, mbw))
            continue
        k = int(rng.integers(cfg.blobs[0], cfg.blobs[1] + 1))
        m = np.zeros((mbh, mbw))
        for _ in range(k):
            cx, cy = rng.uniform(0, mbw), rng.uniform(0, mbh)
            sig = rng.uniform(2.0, 6.0)
            amp = float(rng.lognormal(0.0, 1.0)) if cfg.lognormal_amp else 1.0
            m += amp * np.exp(-((xx - cx) ** 2 + (yy - cy) ** 2) / (2 * sig * sig))
        imp[f] = m + rng.uniform(0.0, 0.1, size=(mbh, mbw))
    if cfg.quantize_levels > 0:
        q = cfg.quantize_levels
        top = max(float(imp.max()), 1e-9)
        imp = np.minimum(np.floor(imp / top * q), q - 1)
    return imp.astype(np.float32)


def make_segments(cfg: Config, n_frames: int | None = None) -> np.ndarray:
    """Selection segments, uint32 [nseg, 3] = (frame_begin, frame_end, k).

    One segment covering the whole batch is the paper's cross-stream queue
    (Sec. 3.3.1); with frac_range set there is one segment per stream with its
    own drawn fraction.  k = floor(frac * macroblocks in the segment).
    """
    F = cfg.n_frames if n_frames is None else n_frames
    per = cfg.mbw * cfg.mbh
    if cfg.frac_range is None:
        return np.array([[0, F, int(np.floor(cfg.frac * F * per + 1e-9))]], dtype=np.uint32)
    rng = np.random.Generator(np.random.PCG64(55_000 + cfg.index))
    fps = F // cfg.n_streams
    segs = []
    for s in range(cfg.n_streams):
        fr = rng.uniform(*cfg.frac_range)
        segs.append([s * fps, (s + 1) * fps, int(np.floor(fr * fps * per))])
    return np.array(segs, dtype=np.uint32)


def make_residuals(width: int, height: int, n_streams: int, frames_per_stream: int, seed: int = 0,
                   noise_sigma: float = 3.0, n_objects=(2, 8), scene_change_prob: float = 0.05) -> np.ndarray:
    """Synthetic luma residuals of decoded chunks, int16 [n_streams * frames_per_stream, H, W].

    Stands in for the codec's Y residual of the paper's 360p streams (Sec. 3.2.2), which are not
    available: low-amplitude noise everywhere (quantisation error), a few small moving objects
    per stream whose residual is strong where they moved (rectangles of 3..40 pixels a side that
    drift, appear and vanish over the chunk), now and then a frame in which a large part of the
    picture changes (a cut or a pan), and isolated strong pixels.  Streams differ in how busy
    they are.  Holds none of the method's arithmetic.
    """
    rng = np.random.Generator(np.random.PCG64(77_000 + seed))
    F = n_streams * frames_per_stream
    res = np.rint(rng.normal(0.0, noise_sigma, size=(F, height, width))).astype(np.int16)
    for s in range(n_streams):
        k = int(rng.integers(n_objects[0], n_objects[1] + 1))
        pos = rng.uniform([0, 0], [width, height], size=(k, 2))
        vel = rng.normal(0.0, 2.0 + 3.0 * rng.random(), size=(k, 2))
        size = rng.integers(3, 41, size=(k, 2))
        alive = rng.random(k) < 0.7
        for t in range(frames_per_stream):
            f = s * frames_per_stream + t
            flip = rng.random(k) < 0.08
            alive = np.where(flip, ~alive, alive)
            pos = (pos + vel) % [width, height]
            for j in range(k):
                if not alive[j]:
                    continue
                x0, y0 = int(pos[j, 0]), int(pos[j, 1])
                x1, y1 = min(width, x0 + int(size[j, 0])), min(height, y0 + int(size[j, 1]))
                amp = rng.integers(25, 90)
                tex = rng.random((y1 - y0, x1 - x0)) < 0.85          # objects are not solid masks
                res[f, y0:y1, x0:x1] += (tex * amp * rng.choice([-1, 1])).astype(np.int16)
            if rng.random() < scene_change_prob:
                y0 = int(rng.integers(0, height // 2)); x0 = int(rng.integers(0, width // 2))
                res[f, y0:y0 + height // 2, x0:x0 + width // 2] += np.int16(rng.integers(30, 70))
            n_hot = int(rng.integers(0, 30))
            ys, xs = rng.integers(0, height, n_hot), rng.integers(0, width, n_hot)
            res[f, ys, xs] += np.int16(60)
    return np.clip(res, -255, 255).astype(np.int16)
