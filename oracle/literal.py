"""Literal fp64 NumPy evaluation of the paper's equations -- TEST INFRASTRUCTURE ONLY.

A second, independent statement of Eq. 1 (Section 3.2) and Eq. 2-3 (Section 3.3)
exactly as printed: exp of the raw logit, no max subtraction, division by the
size-weighted sum, then `S_i > T`.  It is the brute-force check of the C oracle
on small inputs, and it decides which clusters sit so close to the threshold
that an fp32 evaluation may legitimately land on either side.

Pins: tests/test_oracle_scores.py (library softmax for C = L, closed forms).
"""
from __future__ import annotations

import numpy as np

NEAR_BAND = 1e-5   # |ln S_i - ln T| below which a cluster counts as "next to the threshold"


def scores(q, centroids, sizes, sm_scale) -> np.ndarray:
    """Eq. 1: S_i = exp(q.C_i) / sum_j N_j exp(q.C_j), logits scaled by sm_scale.  q [nq,d] -> S [nq,C]."""
    q = np.asarray(q, dtype=np.float64)
    c = np.asarray(centroids, dtype=np.float64)
    n = np.asarray(sizes, dtype=np.float64)
    e = np.exp(np.float64(sm_scale) * (q @ c.T))
    return e / (e * n[None, :]).sum(axis=1, keepdims=True)


def select(q, centroids, sizes, thresh, sm_scale):
    """Kept clusters of one head: boolean [nq, C] (S_i > T, clusters with no keys never kept)."""
    S = scores(q, centroids, sizes, sm_scale)
    return (S > np.float64(thresh)) & (np.asarray(sizes)[None, :] > 0), S


def select_mean(q, centroids, sizes, thresh, sm_scale):
    """Prefill rule of Appendix D for one head: Eq. 1 per query token, averaged over the tokens, then > T.
    q [Lq,d] -> (kept [C] bool, mean scores [C])."""
    Sbar = scores(q, centroids, sizes, sm_scale).mean(axis=0)
    return (Sbar > np.float64(thresh)) & (np.asarray(sizes) > 0), Sbar


def near_threshold(S, thresh, band: float = NEAR_BAND) -> np.ndarray:
    """Clusters whose score is within `band` of the threshold in the log domain."""
    S = np.asarray(S, dtype=np.float64)
    T = np.float64(thresh)
    if T <= 0:
        return np.zeros(S.shape, dtype=bool)
    with np.errstate(divide="ignore"):
        return np.abs(np.log(S) - np.log(T)) <= band


def hier_select(q, centroids1, sizes1, child_offsets, T1, centroids2, sizes2, T2, sm_scale):
    """Eq. 2 then Eq. 3 for ONE query q [d] of one head.

    Returns (keep1 [C1] bool, keep2 [C2] bool, S1 [C1], S2 [C2] with NaN outside the candidates).
    """
    q = np.asarray(q, dtype=np.float64)[None]
    keep1, S1 = select(q, centroids1, sizes1, T1, sm_scale)
    keep1, S1 = keep1[0], S1[0]
    C2 = len(sizes2)
    cand = np.zeros(C2, dtype=bool)
    for j in np.flatnonzero(keep1):
        cand[child_offsets[j]:child_offsets[j + 1]] = True
    S2 = np.full(C2, np.nan)
    keep2 = np.zeros(C2, dtype=bool)
    idx = np.flatnonzero(cand)
    if len(idx):
        k2, s2 = select(q, np.asarray(centroids2)[idx], np.asarray(sizes2)[idx], T2, sm_scale)
        S2[idx] = s2[0]
        keep2[idx] = k2[0]
    return keep1, keep2, S1, S2


def hier_select_mean(q, centroids1, sizes1, child_offsets, T1, centroids2, sizes2, T2, sm_scale):
    """The prefill rule of Appendix D applied level by level (Section 3.3) for one head, q [Lq, d]: the coarse
    scores of Eq. 2 averaged over the query tokens pick the coarse clusters; the fine scores of Eq. 3 -- per token,
    normalised over the children of the kept coarse clusters only -- are averaged over the tokens and compared with T2.
    Returns (keep1 [C1] bool, keep2 [C2] bool, mean S1 [C1], mean S2 [C2] with NaN outside the candidates)."""
    keep1, S1 = select_mean(q, centroids1, sizes1, T1, sm_scale)
    C2 = len(sizes2)
    cand = np.zeros(C2, dtype=bool)
    for j in np.flatnonzero(keep1):
        cand[child_offsets[j]:child_offsets[j + 1]] = True
    S2 = np.full(C2, np.nan)
    keep2 = np.zeros(C2, dtype=bool)
    idx = np.flatnonzero(cand)
    if len(idx):
        k2, s2 = select_mean(q, np.asarray(centroids2)[idx], np.asarray(sizes2)[idx], T2, sm_scale)
        S2[idx] = s2
        keep2[idx] = k2
    return keep1, keep2, S1, S2


def dense_attention(q, K, V, sm_scale):
    """Textbook softmax(sm_scale * q K^T) V for one query set: q [nq,d], K,V [n,d] -> out [nq,d], lse [nq]."""
    q = np.asarray(q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    s = np.float64(sm_scale) * (q @ K.T)
    M = s.max(axis=1, keepdims=True)
    p = np.exp(s - M)
    z = p.sum(axis=1, keepdims=True)
    return (p / z) @ V, (M + np.log(z))[:, 0]


def multilevel_select(q, levels, sm_scale):
    """Section 3.3 level after level for ONE query q [d] of one head, any number of levels, coarsest first.

    levels = list of (centroids [C,d], sizes [C], child_offsets [C+1], T).  Returns per level (keep [C] bool,
    S [C] with NaN outside the level's candidates): at level 0 every cluster is a candidate, below it the children
    of the clusters kept one level up, and Eq. 3's normaliser runs over the candidates only.
    """
    q = np.asarray(q, dtype=np.float64)[None]
    out = []
    cand = np.ones(len(levels[0][1]), dtype=bool)
    for k, (cent, sizes, child_offsets, T) in enumerate(levels):
        Ck = len(sizes)
        S = np.full(Ck, np.nan)
        keep = np.zeros(Ck, dtype=bool)
        idx = np.flatnonzero(cand)
        if len(idx):
            kk, ss = select(q, np.asarray(cent)[idx], np.asarray(sizes)[idx], T, sm_scale)
            S[idx] = ss[0]
            keep[idx] = kk[0]
        out.append((keep, S))
        if k + 1 < len(levels):
            cand = np.zeros(len(levels[k + 1][1]), dtype=bool)
            for j in np.flatnonzero(keep):
                cand[child_offsets[j]:child_offsets[j + 1]] = True
    return out
