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


def mann_whitney_z(a, b) -> dict:
    """Two-sided Mann-Whitney U comparison of two latency samples (paper, appendix "Additional
    Evaluation": configurations are called different when |Z| > 1.96 at significance 0.05).

    Straight from the definition: U_a = #{(i, j): a_i > b_j} + 0.5 * #{(i, j): a_i == b_j};
    normal approximation with the tie-corrected variance and a 0.5 continuity correction
    (the paper names neither; this is the common textbook form):
    mu = n*m/2, sigma^2 = n*m/12 * ((N + 1) - sum(t^3 - t) / (N * (N - 1))), N = n + m,
    t = sizes of the groups of equal values in the pooled sample,
    z = (U_a - mu -/+ 0.5) / sigma (towards zero), z = 0 when U_a == mu or sigma == 0.
    """
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    n, m = len(a), len(b)
    u = 0.0
    for x in a:                                  # pairwise, no ranking shortcut
        u += float((x > b).sum()) + 0.5 * float((x == b).sum())
    big_n = n + m
    _, counts = np.unique(np.concatenate([a, b]), return_counts=True)
    ties = float(((counts.astype(np.float64) ** 3) - counts).sum())
    mu = n * m / 2.0
    var = n * m / 12.0 * ((big_n + 1) - ties / (big_n * (big_n - 1))) if big_n > 1 else 0.0
    d = u - mu
    if var <= 0.0 or d == 0.0:
        z = 0.0
    else:
        z = (d - 0.5 * np.sign(d)) / np.sqrt(var)
    return {"u": u, "z": float(z), "significant": bool(abs(z) > 1.96)}
