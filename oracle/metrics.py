"""Latency determinism metrics of the paper's Section V-A.

On the per-frame end-to-end latencies (arrival at the first stage to departure from the
last), after discarding warm-up and cool-down frames (Section VI: first and last 10 of
1000): mean, maximum, standard deviation, distribution tail (100th minus 95th
percentile) and distribution flatness (90th minus 10th percentile).

Readings where the paper is silent: percentiles interpolate linearly between closest
ranks; the standard deviation is the population one; runs shorter than the paper's
drop min(10, n // 6) frames from each end.
"""
from __future__ import annotations

import numpy as np


def trim_count(n: int) -> int:
    return min(10, n // 6)


def _percentile(sorted_vals: np.ndarray, p: float) -> float:
    n = len(sorted_vals)
    pos = (n - 1) * p / 100.0
    lo = int(np.floor(pos))
    hi = min(lo + 1, n - 1)
    return float(sorted_vals[lo] + (sorted_vals[hi] - sorted_vals[lo]) * (pos - lo))


def determinism_metrics(latencies, trim: bool = True) -> dict:
    x = np.asarray(latencies, dtype=np.float64)
    if trim:
        t = trim_count(len(x))
        x = x[t:len(x) - t]
    s = np.sort(x)
    pct = {p: _percentile(s, p) for p in (10, 50, 90, 95, 99, 100)}
    mean = float(s.sum() / len(s))
    std = float(np.sqrt(((s - mean) ** 2).sum() / len(s)))
    return {"n": int(len(s)), "mean": mean, "max": pct[100], "std": std,
            "p50": pct[50], "p99": pct[99], "tail": pct[100] - pct[95],
            "flatness": pct[90] - pct[10]}
