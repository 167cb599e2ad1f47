"""Exhaustive split search from raw rows -- TEST INFRASTRUCTURE (tiny inputs only).

Sec. 3.1 finds the best split by testing every (feature id, threshold) pair.
Restricted to the k bin boundaries of Sec. 3.3 that is: for every feature and
every boundary, physically partition the leaf's rows, sum the raw gradients and
hessians of each side, and score the partition.  No histogram is ever formed,
so this checks the histogram route (build, then prefix scan) end to end.
"""
from __future__ import annotations

import numpy as np


def brute_force_best_split(bins, n_bins, grad, hess, rows, lam, min_child_hess):
    """Returns (feature, bin, gain) or (-1, -1, 0.0); ties -> smallest feature, then bin."""
    bins = np.asarray(bins)
    rows = np.asarray(rows, dtype=np.int64)
    g = np.asarray(grad, dtype=np.float64)[rows]
    h = np.asarray(hess, dtype=np.float64)[rows]
    G, H = g.sum(), h.sum()
    best = (-1, -1, 0.0)
    have = False
    for f in range(bins.shape[1]):
        col = bins[rows, f].astype(np.int64)
        for t in range(n_bins - 1):
            left = col <= t
            n_l = int(left.sum())
            n_r = int(rows.size - n_l)
            if n_l < 1 or n_r < 1:
                continue
            g_l, h_l = g[left].sum(), h[left].sum()
            g_r, h_r = g[~left].sum(), h[~left].sum()
            if h_l < min_child_hess or h_r < min_child_hess:
                continue
            gain = g_l * g_l / (h_l + lam) + g_r * g_r / (h_r + lam) - G * G / (H + lam)
            if not have or gain > best[2]:
                have = True
                best = (f, t, float(gain))
    return best


def gain_table_from_rows(bins, n_bins, grad, hess, rows, lam, min_child_hess):
    """[n_features, n_bins] gains (NaN where inadmissible), same route as above."""
    bins = np.asarray(bins)
    rows = np.asarray(rows, dtype=np.int64)
    g = np.asarray(grad, dtype=np.float64)[rows]
    h = np.asarray(hess, dtype=np.float64)[rows]
    G, H = g.sum(), h.sum()
    out = np.full((bins.shape[1], n_bins), np.nan)
    for f in range(bins.shape[1]):
        col = bins[rows, f].astype(np.int64)
        for t in range(n_bins - 1):
            left = col <= t
            n_l = int(left.sum())
            n_r = int(rows.size - n_l)
            if n_l < 1 or n_r < 1:
                continue
            g_l, h_l = g[left].sum(), h[left].sum()
            g_r, h_r = g[~left].sum(), h[~left].sum()
            if h_l < min_child_hess or h_r < min_child_hess:
                continue
            out[f, t] = g_l * g_l / (h_l + lam) + g_r * g_r / (h_r + lam) - G * G / (H + lam)
    return out
