"""Stage 1 oracle: format conversion = bilinear resize + uint8 -> float normalise.

Paper, Section III-A: the format-converter operator changes the element datatype of
the frame tensor as pre-processing for inference.  The paper gives no arithmetic; the
reading taken here (exact-rational bilinear with half-pixel centres, one rounding,
then a 256-entry table to float) is listed in the design notes.
"""
from __future__ import annotations

import numpy as np


def _axis_taps(n_in: int, n_out: int):
    """Source taps along one axis.  Sample position of output i is
    (i + 0.5) * n_in / n_out - 0.5, held as the exact rational num / den with
    den = 2 * n_out, clamped to [0, n_in - 1]."""
    i = np.arange(n_out, dtype=np.int64)
    den = 2 * n_out
    num = (2 * i + 1) * n_in - n_out
    num = np.clip(num, 0, (n_in - 1) * den)
    i0 = num // den
    frac = num % den
    i1 = np.minimum(i0 + 1, n_in - 1)
    return i0, i1, frac, den


def resize_bilinear_u8(frame: np.ndarray, w_out: int, h_out: int) -> np.ndarray:
    """Bilinear resample of an (H, W, C) uint8 image to (h_out, w_out, C) uint8.

    The four-tap weighted sum is formed exactly in integers and rounded once,
    half-up: q = floor((acc + D/2) / D), D = (2*w_out) * (2*h_out).
    """
    assert frame.dtype == np.uint8 and frame.ndim == 3
    h_in, w_in, _ = frame.shape
    x0, x1, fx, dx = _axis_taps(w_in, w_out)
    y0, y1, fy, dy = _axis_taps(h_in, h_out)
    p = frame.astype(np.int64)
    wx1 = fx[None, :, None]
    wx0 = dx - wx1
    wy1 = fy[:, None, None]
    wy0 = dy - wy1
    p00 = p[y0][:, x0]
    p01 = p[y0][:, x1]
    p10 = p[y1][:, x0]
    p11 = p[y1][:, x1]
    acc = wx0 * wy0 * p00 + wx1 * wy0 * p01 + wx0 * wy1 * p10 + wx1 * wy1 * p11
    d = dx * dy
    q = (acc + d // 2) // d
    return q.astype(np.uint8)


def normalize_lut(mean: float, std: float, fp16: bool) -> np.ndarray:
    """LUT[v] = float32((v / 255 - mean) / std) for v in 0..255, evaluated in float64.
    With ``fp16`` the float32 entry is further rounded (nearest-even) to half precision;
    the table is returned as float32 either way."""
    v = np.arange(256, dtype=np.float64)
    lut = ((v / 255.0 - np.float64(np.float32(mean))) / np.float64(np.float32(std)))
    lut = lut.astype(np.float32)
    if fp16:
        lut = lut.astype(np.float16).astype(np.float32)
    return lut


def preprocess(frame: np.ndarray, w_out: int, h_out: int, mean: float, std: float,
               fp16: bool):
    """Full stage 1: returns (resized uint8 HWC, normalised planar CHW float32)."""
    q = resize_bilinear_u8(frame, w_out, h_out)
    lut = normalize_lut(mean, std, fp16)
    planar = np.ascontiguousarray(lut[q].transpose(2, 0, 1))
    return q, planar
