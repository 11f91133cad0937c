"""Seeded synthetic frames standing in for traffic-camera video.

make_frames(scene, seed) -> uint8 [n_frames, 3, H, W].

"road" style: a gray road (level 100-130) with mild low-frequency shading;
`rect_min..rect_max` solid axis-aligned rectangles (vehicle-like aspect 0.5-2.5,
longer side `side_min..side_max` px), each moving along a fixed heading by a few
pixels per frame with +-1 px jitter, so consecutive frames are correlated.
"gradient" style: a per-channel linear + cosine gradient background with static
rectangles re-drawn per frame with fresh positions.

The number of rectangles of a sequence is drawn once; rectangle r of frame t is a
pure function of (seed, r, t).  `scene.noise` > 0 adds per-pixel, per-channel sensor
noise (uniform integers in -noise .. +noise, a pure function of (seed, t, position))
on top of the drawn frame, as a camera would.
"""
import numpy as np

from . import rng
from .configs import SceneSpec


def _background(scene: SceneSpec, seed: int):
    H, W = scene.height, scene.width
    y = np.arange(H, dtype=np.float64)[:, None] / H
    x = np.arange(W, dtype=np.float64)[None, :] / W
    p = rng.uniform(seed, 1, 16)
    bg = np.empty((3, H, W), dtype=np.float64)
    if scene.style == "road":
        base = 100.0 + 30.0 * p[0]
        shade = 8.0 * np.cos(2 * np.pi * (p[1] * x + p[2] * y + p[3])) + 5.0 * np.cos(2 * np.pi * (1.7 * p[4] * x - 1.3 * p[5] * y))
        for c in range(3):
            bg[c] = base + shade + 3.0 * (p[6 + c] - 0.5)
    else:
        for c in range(3):
            bg[c] = (60.0 + 120.0 * p[c] + 50.0 * (p[3 + c] - 0.5) * x + 50.0 * (p[6 + c] - 0.5) * y
                     + 20.0 * np.cos(2 * np.pi * (p[9 + c] * x + p[12 + c] * y)))
    return bg


def make_frames(scene: SceneSpec, seed: int, n_frames=None) -> np.ndarray:
    H, W = scene.height, scene.width
    n = scene.n_frames if n_frames is None else n_frames
    bg = np.clip(np.rint(_background(scene, seed)), 0, 255).astype(np.uint8)
    n_rect = int(rng.randint(seed, 2, scene.rect_min, scene.rect_max, 1)[0])
    u = rng.uniform(seed, 3, 12 * n_rect).reshape(n_rect, 12)
    frames = np.empty((n, 3, H, W), dtype=np.uint8)
    for t in range(n):
        img = bg.copy()
        jit = rng.randint(seed, 4, -1, 1, 2 * n_rect, 2 * n_rect * t).reshape(n_rect, 2)
        if scene.style != "road":
            ut = rng.uniform(seed, 5, 2 * n_rect, 2 * n_rect * t).reshape(n_rect, 2)
        for r in range(n_rect):
            long_side = scene.side_min + u[r, 0] * (scene.side_max - scene.side_min)
            aspect = 0.5 + 2.0 * u[r, 1]                       # w / h in 0.5 .. 2.5
            if aspect >= 1.0:
                w, h = long_side, long_side / aspect
            else:
                w, h = long_side * aspect, long_side
            w, h = max(2, int(w)), max(2, int(h))
            if scene.style == "road":
                ang = 2 * np.pi * u[r, 4]
                speed = 1.0 + 3.0 * u[r, 5]
                cx = u[r, 2] * W + speed * np.cos(ang) * t + jit[r, 0]
                cy = u[r, 3] * H + speed * np.sin(ang) * t + jit[r, 1]
                cx, cy = cx % W, cy % H
            else:
                cx, cy = ut[r, 0] * W, ut[r, 1] * H
            x0, y0 = int(cx - w / 2), int(cy - h / 2)
            x1, y1 = x0 + w, y0 + h
            x0, y0, x1, y1 = max(x0, 0), max(y0, 0), min(x1, W), min(y1, H)
            if x1 <= x0 or y1 <= y0:
                continue
            for c in range(3):
                img[c, y0:y1, x0:x1] = int(255 * u[r, 6 + c])
        if scene.noise > 0:
            a = int(scene.noise)
            nb = 3 * H * W
            raw = rng.bits64(seed, 6, t * ((nb + 7) // 8), (nb + 7) // 8).view(np.uint8)[:nb].reshape(3, H, W)
            img = np.clip(img.astype(np.int16) + (raw % (2 * a + 1)).astype(np.int16) - a, 0, 255).astype(np.uint8)
        frames[t] = img
    return frames
