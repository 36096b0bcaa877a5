"""Stage 3 oracle: tool-tracking postprocess of the network's logits.

Paper, Section III-A: a postprocessor turns the inference output into a tool
segmentation.  No arithmetic is given; the reading here: per channel, heat =
sigmoid(logit), mask = heat > threshold, one peak position per channel.  The integer
outputs are decided on the logits with exact comparisons (sigmoid is strictly
monotone, so heat > t  <=>  logit > ln(t / (1 - t))), which avoids spurious ties from
a rounded sigmoid.
"""
from __future__ import annotations

import numpy as np


def logit_threshold(t: float) -> np.float32:
    """theta = ln(t / (1 - t)) in float64, rounded to float32 (t = 0.5 -> exactly 0)."""
    t = np.float64(np.float32(t))
    return np.float32(np.log(t / (1.0 - t)))


def postprocess(logits: np.ndarray, threshold: float):
    """logits: (K, H, W) float32.  Returns dict with
    heat (K,H,W) float32, mask (K,H,W) uint8, argmax_idx (K,) int32 (row-major,
    lowest index among equal maxima), present (K,) uint8, peak (K,) float32."""
    logits = np.asarray(logits, dtype=np.float32)
    k = logits.shape[0]
    theta = logit_threshold(threshold)
    heat = (1.0 / (1.0 + np.exp(-logits.astype(np.float64)))).astype(np.float32)
    mask = (logits > theta).astype(np.uint8)
    flat = logits.reshape(k, -1)
    argmax_idx = np.zeros(k, dtype=np.int32)
    best = np.zeros(k, dtype=np.float32)
    for ch in range(k):
        b, bi = flat[ch, 0], 0
        for i in range(1, flat.shape[1]):
            if flat[ch, i] > b:          # strict: the lowest index wins ties
                b, bi = flat[ch, i], i
        argmax_idx[ch], best[ch] = bi, b
    peak = (1.0 / (1.0 + np.exp(-best.astype(np.float64)))).astype(np.float32)
    present = (best > theta).astype(np.uint8)
    return {"heat": heat, "mask": mask, "argmax_idx": argmax_idx, "present": present,
            "peak": peak}
