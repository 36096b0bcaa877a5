"""Synthetic RGB uint8 video frames standing in for the endoscopy sample video.

The paper replays a recorded endoscopy video (Section V-B, "Applications"); that
video is not available, so frames of the same shape (HWC, RGB, uint8) are generated:

* ``uniform_frames``: i.i.d. uniform bytes (small smoke/parity configuration).
* ``tool_scene_frames``: a smooth colour gradient, three moving grey rectangles that
  play the role of surgical tools, and additive Gaussian noise (sigma 10).
"""
from __future__ import annotations

import numpy as np

# eight overlay colours, one per tool channel (RGB)
DEFAULT_PALETTE = np.array(
    [(255, 0, 0), (0, 255, 0), (0, 0, 255), (255, 255, 0),
     (255, 0, 255), (0, 255, 255), (255, 128, 0), (255, 255, 255)], dtype=np.uint8)


def uniform_frames(n: int, h: int, w: int, seed: int) -> np.ndarray:
    """``n`` frames of shape (h, w, 3), every byte uniform in [0, 255]."""
    rng = np.random.default_rng([seed, 1])
    return rng.integers(0, 256, size=(n, h, w, 3), dtype=np.uint8)


def tool_scene_frames(n: int, h: int, w: int, seed: int, sigma: float = 10.0):
    """Generator of ``n`` frames (h, w, 3) uint8: gradient + 3 grey rectangles + noise.

    Rectangles: width U[w/16, w/4], height U[h/45, h/11.25] (120..480 x 24..96 at
    1080p), grey level U[150, 230], start position uniform inside the frame, velocity
    U[-8, 8] px/frame per axis, reflected at the borders, drawn in index order.
    """
    rng = np.random.default_rng([seed, 2])
    xs = np.arange(w, dtype=np.float32)[None, :]
    ys = np.arange(h, dtype=np.float32)[:, None]
    base = np.empty((h, w, 3), dtype=np.float32)
    base[..., 0] = 255.0 * xs / max(w - 1, 1)
    base[..., 1] = 255.0 * ys / max(h - 1, 1)
    base[..., 2] = 255.0 * (xs + ys) / max(w + h - 2, 1)
    n_rect = 3
    rw = rng.uniform(w / 16.0, w / 4.0, n_rect)
    rh = rng.uniform(h / 45.0, h / 11.25, n_rect)
    grey = rng.uniform(150.0, 230.0, n_rect)
    px = rng.uniform(0.0, 1.0, n_rect) * (w - rw)
    py = rng.uniform(0.0, 1.0, n_rect) * (h - rh)
    vx = rng.uniform(-8.0, 8.0, n_rect)
    vy = rng.uniform(-8.0, 8.0, n_rect)
    for _ in range(n):
        img = base.copy()
        for r in range(n_rect):
            x0, y0 = int(px[r]), int(py[r])
            x1, y1 = min(w, x0 + int(rw[r])), min(h, y0 + int(rh[r]))
            img[y0:y1, x0:x1, :] = np.float32(grey[r])
        img += rng.standard_normal(img.shape, dtype=np.float32) * np.float32(sigma)
        yield np.clip(np.rint(img), 0, 255).astype(np.uint8)
        px += vx
        py += vy
        for r in range(n_rect):
            if px[r] < 0 or px[r] > w - rw[r]:
                vx[r] = -vx[r]
                px[r] = min(max(px[r], 0.0), w - rw[r])
            if py[r] < 0 or py[r] > h - rh[r]:
                vy[r] = -vy[r]
                py[r] = min(max(py[r], 0.0), h - rh[r])
