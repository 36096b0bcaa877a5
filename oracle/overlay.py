"""Stage 4 oracle: overlay of the tool masks on the ORIGINAL full-resolution frame.

Paper, Sections II-B and III-A: the visualisation operator draws the segmented tools
over the original input frame.  Done here as plain integer compositing: nearest
(floor) upsampling of the masks, lowest set channel wins, Q8 alpha blend.
"""
from __future__ import annotations

import numpy as np


def alpha_q8(alpha: float) -> int:
    """a = clamp(round-half-even(256 * alpha), 0, 256); 256 means opaque."""
    return int(min(256, max(0, int(np.rint(256.0 * np.float64(np.float32(alpha)))))))


def overlay(frame: np.ndarray, mask: np.ndarray, palette: np.ndarray, alpha: float):
    """frame (Hf, Wf, 3) uint8; mask (K, Hm, Wm) of {0,1}; palette (K, 3) uint8.
    Pixel (X, Y) looks at mask cell (floor(X*Wm/Wf), floor(Y*Hm/Hf)); if channel k* is
    the lowest channel set there, out = (a*pal[k*] + (256-a)*in + 128) >> 8, else in."""
    hf, wf, _ = frame.shape
    k, hm, wm = mask.shape
    a = alpha_q8(alpha)
    mx = (np.arange(wf, dtype=np.int64) * wm) // wf
    my = (np.arange(hf, dtype=np.int64) * hm) // hf
    up = mask[:, my][:, :, mx] != 0                       # (K, Hf, Wf)
    any_set = up.any(axis=0)
    kstar = np.argmax(up, axis=0)                         # first True = lowest channel
    colour = palette.astype(np.int64)[kstar]              # (Hf, Wf, 3)
    src = frame.astype(np.int64)
    blended = (a * colour + (256 - a) * src + 128) >> 8
    out = np.where(any_set[..., None], blended, src)
    return out.astype(np.uint8)
