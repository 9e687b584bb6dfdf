"""Byte accounting of the method: what one decode step must move, and the paper's "KV budget".

KV budget (Appendix "KV Budget Computation", Table "LongBench evaluation"): the expected fraction of the KV
cache bytes loaded, including the centroids.  Centroids exist for keys only, so a centroid count of `c`
(as a fraction of the context length) costs c/2 of the K+V bytes; with a two-level lookup only the coarse
centroids and the fine centroids under kept coarse clusters are loaded.
"""
from __future__ import annotations

import numpy as np


def kv_budget(sparsity: float, centroid_frac: float) -> float:
    """One-level: (1 - sparsity) of the keys and values, plus centroids (keys only)."""
    return (1.0 - sparsity) + centroid_frac / 2.0


def centroid_overhead(centroid_frac1: float, centroid_frac2: float = 0.0, coarse_keep: float = 1.0):
    """(stored, loaded) centroid bytes as a fraction of the K+V bytes for a one- or two-level lookup."""
    if centroid_frac2 == 0.0:
        return centroid_frac1 / 2.0, centroid_frac1 / 2.0
    return (centroid_frac1 + centroid_frac2) / 2.0, (centroid_frac1 + coarse_keep * centroid_frac2) / 2.0


def decode_step_bytes(H, C, d, U, B, n_keys_per_row):
    """Algorithmic HBM bytes of one decode step for the achieved selection (fp16 storage)."""
    centroid = H * C * d * 2
    meta = H * C * 4 + H * (C + 1) * 4 + H * 4
    selected_kv = int(np.sum(n_keys_per_row)) * d * 2 * 2
    dense_kv = B * H * U * d * 2 * 2
    io = B * H * d * 2 * 2
    return dict(centroid=centroid, meta=meta, selected_kv=selected_kv, dense_kv=dense_kv, io=io,
                total=centroid + meta + selected_kv + dense_kv + io)
