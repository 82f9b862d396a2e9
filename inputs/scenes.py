"""Seeded moving-camera frame sequences for the five synthetic workloads.

Every sequence is a crop window sliding over a static "panorama" (a sum of
Gaussian blobs per channel) with a few moving objects and per-frame sensor
noise; the camera moves by whole tiles (tile = total network stride), so the
per-frame shift handed to the method is an integer number of tiles.  Frames
are NHWC in the network's storage dtype.  Nothing here depends on the method.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np

from .nets import BASE_SEED


@dataclass
class Sequence:
    frames: np.ndarray                 # [T, H, W, C] storage dtype
    shifts: np.ndarray                 # [T, 2] int32: (dty, dtx) in tiles, applied before frame t
    forced: Optional[np.ndarray]       # [T, H, W] uint8 forced input masks, or None
    tile: int                          # input pixels per tile


def _rng(config: int, stream: int = 0) -> np.random.Generator:
    return np.random.default_rng(np.random.PCG64(BASE_SEED + config + 1000 * stream))


def blob_field(rng, C, H, W, n_blobs=40, sigma=(4.0, 12.0)) -> np.ndarray:
    """[H, W, C] float32: per channel the sum of n_blobs separable Gaussians."""
    out = np.empty((H, W, C), np.float32)
    ys = np.arange(H, dtype=np.float64)[None, :]
    xs = np.arange(W, dtype=np.float64)[None, :]
    for c in range(C):
        cy = rng.uniform(0, H, n_blobs)[:, None]
        cx = rng.uniform(0, W, n_blobs)[:, None]
        sg = rng.uniform(sigma[0], sigma[1], n_blobs)[:, None]
        amp = rng.uniform(-1.0, 1.0, n_blobs)[:, None]
        gy = np.exp(-0.5 * ((ys - cy) / sg) ** 2)
        gx = np.exp(-0.5 * ((xs - cx) / sg) ** 2) * amp
        out[:, :, c] = (gy.T @ gx).astype(np.float32)
    return out


def _paste(dst, patch, y, x):
    """Overwrite dst[y:y+h, x:x+w] with patch, clipped to dst."""
    H, W = dst.shape[:2]
    h, w = patch.shape[:2]
    y0, x0 = max(y, 0), max(x, 0)
    y1, x1 = min(y + h, H), min(x + w, W)
    if y1 > y0 and x1 > x0:
        dst[y0:y1, x0:x1] = patch[y0 - y:y1 - y, x0 - x:x1 - x]


def _finish(frames, pos, tile, dtype, forced=None) -> Sequence:
    pos = np.asarray(pos, np.int64)
    d = np.zeros_like(pos)
    d[1:] = pos[1:] - pos[:-1]
    assert np.all(d % tile == 0)
    return Sequence(np.stack(frames).astype(dtype), (d // tile).astype(np.int32), forced, tile)


def _seq1(n_frames=3, H=64, W=64, C=16, step=(2, 3)) -> Sequence:
    rng = _rng(1)
    pano = blob_field(rng, C, 2 * H, 2 * W)
    frames, pos = [], []
    for t in range(n_frames):
        y, x = step[0] * t, step[1] * t
        sy = y + int(rng.integers(0, H - 8 + 1))
        sx = x + int(rng.integers(0, W - 8 + 1))
        pano[sy:sy + 8, sx:sx + 8] = rng.uniform(-1, 1, (8, 8, C)).astype(np.float32)
        f = pano[y:y + H, x:x + W] + rng.normal(0, 0.01, (H, W, C)).astype(np.float32)
        frames.append(f)
        pos.append((y, x))
    return _finish(frames, pos, 1, np.float32)


def _seq2(n_frames=30, H=256, W=256) -> Sequence:
    rng = _rng(2)
    PH, PW = max(1024, H), max(512, W + 4 * n_frames)
    pano = blob_field(rng, 3, PH, PW)
    y0 = (PH - H) // 2
    rect_p = np.stack([rng.uniform(y0, y0 + H - 24, 3), rng.uniform(0, W - 24, 3)], 1)
    rect_v = rng.uniform(-3, 3, (3, 2))
    rect_c = rng.uniform(-1, 1, (3, 3)).astype(np.float32)
    frames, pos = [], []
    for t in range(n_frames):
        x = 4 * t
        scene = pano.copy()
        for r in range(3):
            p = np.rint(rect_p[r] + t * rect_v[r]).astype(int)
            _paste(scene, np.broadcast_to(rect_c[r], (24, 24, 3)), int(p[0]), int(p[1]))
        f = scene[y0:y0 + H, x:x + W] + rng.normal(0, 0.005, (H, W, 3)).astype(np.float32)
        frames.append(f)
        pos.append((y0, x))
    return _finish(frames, pos, 4, np.float32)


def _seq3(n_frames=60, H=512, W=512, tile=8) -> Sequence:
    rng = _rng(3)
    PH, PW = 4 * H, 4 * W
    pano = blob_field(rng, 3, PH, PW)
    y, x = (PH - H) // 2, (PW - W) // 2
    n_obj = 10
    size = rng.integers(16, 65, n_obj)
    tex = [blob_field(rng, 3, int(s), int(s), n_blobs=6, sigma=(2.0, 6.0)) for s in size]
    p0 = np.stack([rng.uniform(y, y + H, n_obj), rng.uniform(x, x + W, n_obj)], 1)
    vel = rng.uniform(-3, 3, (n_obj, 2))
    frames, pos = [], []
    for t in range(n_frames):
        if t > 0:
            sy, sx = (int(v) * tile for v in rng.integers(-2, 3, 2))
            if not 0 <= y + sy <= PH - H:
                sy = -sy
            if not 0 <= x + sx <= PW - W:
                sx = -sx
            y, x = y + sy, x + sx
        view = pano[y:y + H, x:x + W].copy()
        for o in range(n_obj):
            p = np.rint(p0[o] + t * vel[o]).astype(int)
            _paste(view, tex[o], int(p[0]) - y, int(p[1]) - x)
        view += rng.normal(0, 0.005, (H, W, 3)).astype(np.float32)
        frames.append(view)
        pos.append((y, x))
    return _finish(frames, pos, tile, np.float16)


def _seq4(n_frames=100, H=384, W=288, tile=32) -> Sequence:
    rng = _rng(4)
    PH, PW = 2 * H, 16 * W // 3
    pano = blob_field(rng, 3, PH, PW)
    y, x = (PH - H) // 2, (PW - W) // 2
    n_obj = 20
    p0 = np.stack([rng.uniform(y, y + H, n_obj), rng.uniform(x, x + W, n_obj)], 1)
    vel = rng.uniform(-2, 2, (n_obj, 2))
    sg = rng.uniform(3, 8, n_obj)
    amp = rng.uniform(-1, 1, (n_obj, 3)).astype(np.float32)
    frames, pos = [], []
    direction = 1
    for t in range(n_frames):
        if t > 0 and t % 8 == 0:
            x = int(np.clip(x + direction * tile * int(rng.integers(1, 3)), 0, PW - W))
            direction = -direction
        ys = np.arange(y, y + H, dtype=np.float64)[:, None]
        xs = np.arange(x, x + W, dtype=np.float64)[None, :]
        view = pano[y:y + H, x:x + W].copy()
        for o in range(n_obj):
            c = p0[o] + t * vel[o]
            g = np.exp(-0.5 * (((ys - c[0]) / sg[o]) ** 2 + ((xs - c[1]) / sg[o]) ** 2))
            view += g[:, :, None].astype(np.float32) * amp[o]
        view += rng.normal(0, 0.005, (H, W, 3)).astype(np.float32)
        frames.append(view)
        pos.append((y, x))
    return _finish(frames, pos, tile, np.float16)


def clustered_tile_mask(rng, H, W, density, tile=4) -> np.ndarray:
    """[H, W] uint8 union of tile x tile squares drawn around a few cluster centres
    until the requested fraction of tiles is set."""
    th, tw = H // tile, W // tile
    n_target = int(round(density * th * tw))
    m = np.zeros((th, tw), np.uint8)
    if n_target >= th * tw:
        m[:] = 1
    else:
        n_clusters = max(1, n_target // 24)
        cy = rng.uniform(0, th, n_clusters)
        cx = rng.uniform(0, tw, n_clusters)
        spread = max(1.0, np.sqrt(n_target / n_clusters) * 0.6)
        count = 0
        while count < n_target:
            c = rng.integers(0, n_clusters, 256)
            ty = np.clip(np.rint(cy[c] + rng.normal(0, spread, 256)), 0, th - 1).astype(int)
            tx = np.clip(np.rint(cx[c] + rng.normal(0, spread, 256)), 0, tw - 1).astype(int)
            for a, b in zip(ty, tx):
                if count >= n_target:
                    break
                if not m[a, b]:
                    m[a, b] = 1
                    count += 1
    return np.kron(m, np.ones((tile, tile), np.uint8))


def _seq5(density=0.2, n_frames=50, H=128, W=128, C=256, shift_every=10, shift=16) -> Sequence:
    rng = _rng(5, stream=int(round(density * 1000)))
    n_shifts = (n_frames - 1) // shift_every
    canvas = rng.normal(0, 0.5, (H, W + shift * n_shifts, C)).astype(np.float32).astype(np.float16)
    frames, pos, forced = [], [], []
    x = 0
    for t in range(n_frames):
        if t > 0 and t % shift_every == 0:
            x += shift
        m = clustered_tile_mask(rng, H, W, density)
        view = canvas[:, x:x + W]
        idx = m.astype(bool)
        d = rng.normal(0, 0.1, (int(idx.sum()), C)).astype(np.float32)
        view[idx] = (view[idx].astype(np.float32) + d).astype(np.float16)
        frames.append(view.copy())
        forced.append(m)
        pos.append((0, x))
    return _finish(frames, pos, 1, np.float16, np.stack(forced))


def build_sequence(config: int, **kw) -> Sequence:
    """Frame sequence of benchmark workload `config` (1..5).  Keyword overrides
    (n_frames, H, W, density, ...) give reduced parity cases from the same recipe."""
    return {1: _seq1, 2: _seq2, 3: _seq3, 4: _seq4, 5: _seq5}[config](**kw)
