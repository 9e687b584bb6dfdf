"""Offline clustering of the fixed-context keys (Section 3.1) -- TEST INFRASTRUCTURE ONLY, plain NumPy fp64.

The paper clusters the keys of a head with K-means on NORMALISED key vectors and then takes, per cluster, the
mean of the vectors in it as the centroid the online lookup compares queries with.  It fixes neither the
initialisation nor the number of iterations, so the unit defined here is one Lloyd iteration plus the final
layout step; readings taken: squared Euclidean distance between unit vectors (the usual K-means objective, which
on unit vectors orders centres like cosine similarity corrected by the centre's norm); a centre is the plain mean
of its members' normalised vectors (not re-normalised); a centre that loses all members keeps its value; ties go
to the lowest centre index; the centroid handed to the online path is the per-cluster mean of the RAW keys
(Section 3.1 defines a centroid as the average of its cluster's members), as in the workload generator.

Pins: tests/test_oracle_clustering.py.
"""
from __future__ import annotations

import numpy as np


def normalize_rows(K) -> np.ndarray:
    """k / |k| per row, fp64 arithmetic on the fp16 values, rounded to fp16 (zero rows stay zero)."""
    K = np.asarray(K, dtype=np.float64)
    n = np.sqrt((K * K).sum(axis=-1, keepdims=True))
    return np.where(n > 0, K / np.where(n > 0, n, 1.0), 0.0).astype(np.float16)


def assign(X, centers):
    """Nearest centre of every row: argmin_c |x - c|^2 = argmax_c (x.c - |c|^2 / 2), lowest index on ties.

    X [L, d], centers [C, d] (fp16 values, fp64 arithmetic) -> (assign [L] int32, margin [L] fp64 = score of the best
    centre minus score of the runner-up; small margins mark rows an fp32 evaluation may assign either way)."""
    X = np.asarray(X, dtype=np.float64)
    Cc = np.asarray(centers, dtype=np.float64)
    s = X @ Cc.T - 0.5 * (Cc * Cc).sum(axis=1)[None, :]
    a = np.argmax(s, axis=1)                                   # first maximum = lowest index
    if s.shape[1] > 1:
        top2 = np.partition(s, -2, axis=1)[:, -2:]
        margin = top2[:, 1] - top2[:, 0]
    else:
        margin = np.full(len(X), np.inf)
    return a.astype(np.int32), margin


def update(X, a, centers_prev):
    """Mean of the members of every cluster (fp64), rounded to fp16; a cluster without members keeps its centre.
    -> (centers [C, d] fp16, counts [C] int32)."""
    X = np.asarray(X, dtype=np.float64)
    C, d = np.asarray(centers_prev).shape
    counts = np.bincount(a, minlength=C).astype(np.int32)
    sums = np.zeros((C, d))
    np.add.at(sums, a, X)
    out = np.asarray(centers_prev, dtype=np.float64).copy()
    nz = counts > 0
    out[nz] = sums[nz] / counts[nz, None]
    return out.astype(np.float16), counts


def lloyd_step(X, centers):
    """One Lloyd iteration: assign, then update.  -> (assign, new centers fp16, counts, objective before the update)."""
    a, _ = assign(X, centers)
    Xd = np.asarray(X, dtype=np.float64)
    obj = float(((Xd - np.asarray(centers, dtype=np.float64)[a]) ** 2).sum())
    c, n = update(X, a, centers)
    return a, c, n, obj


def layout(K, a, C):
    """Inputs of the online path from an assignment: keys sorted by cluster id (stable: ascending key index inside a
    cluster), sizes, offsets, and the centroid of every cluster = mean of its RAW keys (fp64 -> fp16; zeros for an
    empty cluster).  -> (perm [L], sizes [C], offsets [C+1], centroids [C, d] fp16)."""
    K = np.asarray(K)
    perm = np.argsort(a, kind="stable").astype(np.int32)
    sizes = np.bincount(a, minlength=C).astype(np.int32)
    offsets = np.zeros(C + 1, np.int32)
    offsets[1:] = np.cumsum(sizes)
    cent = np.zeros((C, K.shape[1]))
    np.add.at(cent, a, K.astype(np.float64))
    nz = sizes > 0
    cent[nz] /= sizes[nz, None]
    return perm, sizes, offsets, cent.astype(np.float16)


def nest(assign_fine, perm_coarse, child_offsets, C2):
    """Fine clusters nested under coarse ones (Section 3.3: the coarse level clusters the fine centroids).
    perm_coarse [C2]: fine ids grouped by coarse cluster; child_offsets [C1+1].  The fine clusters are renumbered in
    perm_coarse order and the keys grouped again.
    -> (assign_new [L], sizes [C2], offsets [C2+1], perm [L], sizes_coarse [C1] keys under each coarse cluster)."""
    perm_coarse = np.asarray(perm_coarse)
    inv = np.empty(C2, np.int64)
    inv[perm_coarse] = np.arange(C2)
    assign_new = inv[np.asarray(assign_fine)].astype(np.int32)
    perm = np.argsort(assign_new, kind="stable").astype(np.int32)
    sizes = np.bincount(assign_new, minlength=C2).astype(np.int32)
    offsets = np.zeros(C2 + 1, np.int32)
    offsets[1:] = np.cumsum(sizes)
    co = np.asarray(child_offsets)
    sizes_coarse = (offsets[co[1:]] - offsets[co[:-1]]).astype(np.int32)
    return assign_new, sizes, offsets, perm, sizes_coarse
