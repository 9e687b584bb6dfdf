"""CPU oracle for the Squeezed Attention online path -- TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's CPU-baseline leg may import
this package.  It is independent of the GPU library: no shared code, headers or
helpers, and neither side imports the other.

`squeezed_oracle.c` holds the step-by-step fp32/fp64 C implementation (built by
`build()` with gcc); `literal.py` holds a second, literal fp64 NumPy evaluation
of Eq. 1-3 used for brute-force checks and for classifying clusters whose score
lies next to the threshold.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional

import numpy as np

_DIR = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_DIR, "squeezed_oracle.c")
_LIB = os.path.join(_DIR, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (plain -O2, OpenMP over (sequence, head, query))."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared",
                               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        _lib.oracle_num_threads.restype = C.c_int
    return _lib


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f16(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    assert a.dtype == np.float16, a.dtype
    return a


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def centroid_score(q, centroids, sizes, sm_scale):
    """q [B,H,Lq,d] f16, centroids [H,C,d] f16, sizes [H,C] -> logits [B,H,Lq,C], row_max, denom [B,H,Lq]."""
    q, centroids, sizes = _f16(q), _f16(centroids), _i32(sizes)
    B, H, Lq, d = q.shape
    Cn = centroids.shape[1]
    assert centroids.shape == (H, Cn, d) and sizes.shape == (H, Cn)
    logits = np.empty((B, H, Lq, Cn), np.float32)
    row_max = np.empty((B, H, Lq), np.float32)
    denom = np.empty((B, H, Lq), np.float32)
    lib().oracle_centroid_score(B, H, Lq, Cn, d, C.c_float(sm_scale), _p(q), _p(centroids), _p(sizes),
                                _p(logits), _p(row_max), _p(denom))
    return logits, row_max, denom


def select(logits, row_max, denom, thresh, sizes, offsets):
    """-> keep_mask [B,H,Lq,ceil(C/32)] u32, ranges [B,H,Lq,C,2] i32, n_ranges, n_keys [B,H,Lq] i32."""
    logits, row_max, denom, thresh = _f32(logits), _f32(row_max), _f32(denom), _f32(thresh)
    sizes, offsets = _i32(sizes), _i32(offsets)
    B, H, Lq, Cn = logits.shape
    assert thresh.shape == (H,) and sizes.shape == (H, Cn) and offsets.shape == (H, Cn + 1)
    W = (Cn + 31) // 32
    mask = np.empty((B, H, Lq, W), np.uint32)
    ranges = np.zeros((B, H, Lq, Cn, 2), np.int32)
    n_ranges = np.empty((B, H, Lq), np.int32)
    n_keys = np.empty((B, H, Lq), np.int32)
    lib().oracle_select(B, H, Lq, Cn, _p(logits), _p(row_max), _p(denom), _p(thresh), _p(sizes), _p(offsets),
                        _p(mask), _p(ranges), _p(n_ranges), _p(n_keys))
    return mask, ranges, n_ranges, n_keys


def select_mean(logits, row_max, denom, thresh, sizes, offsets, want_scores: bool = False):
    """Prefill selection on scores averaged over the Lq query tokens (Appendix D).
    -> keep_mask [B,H,ceil(C/32)] u32, ranges [B,H,C,2] i32, n_ranges, n_keys [B,H] i32 [, mean scores [B,H,C] f64]."""
    logits, row_max, denom, thresh = _f32(logits), _f32(row_max), _f32(denom), _f32(thresh)
    sizes, offsets = _i32(sizes), _i32(offsets)
    B, H, Lq, Cn = logits.shape
    assert thresh.shape == (H,) and sizes.shape == (H, Cn) and offsets.shape == (H, Cn + 1)
    W = (Cn + 31) // 32
    mask = np.empty((B, H, W), np.uint32)
    ranges = np.zeros((B, H, Cn, 2), np.int32)
    n_ranges = np.empty((B, H), np.int32)
    n_keys = np.empty((B, H), np.int32)
    sbar = np.empty((B, H, Cn), np.float64) if want_scores else None
    lib().oracle_select_mean(B, H, Lq, Cn, _p(logits), _p(row_max), _p(denom), _p(thresh), _p(sizes), _p(offsets),
                             _p(mask), _p(ranges), _p(n_ranges), _p(n_keys), _p(sbar))
    return (mask, ranges, n_ranges, n_keys, sbar) if want_scores else (mask, ranges, n_ranges, n_keys)


def hier_select(q, centroids1, sizes1, child_offsets, thresh1, centroids2, sizes2, offsets2, thresh2, sm_scale,
                want_logits2: bool = False):
    """Two-level lookup, q [B,H,1,d] or [B,H,d].  Returns dict(mask1, mask2, ranges, n_ranges, n_keys, stats[, logits2])."""
    q = _f16(q)
    if q.ndim == 4:
        assert q.shape[2] == 1
        q = np.ascontiguousarray(q[:, :, 0])
    B, H, d = q.shape
    centroids1, centroids2 = _f16(centroids1), _f16(centroids2)
    sizes1, child_offsets, sizes2, offsets2 = _i32(sizes1), _i32(child_offsets), _i32(sizes2), _i32(offsets2)
    thresh1, thresh2 = _f32(thresh1), _f32(thresh2)
    C1, C2 = centroids1.shape[1], centroids2.shape[1]
    assert child_offsets.shape == (H, C1 + 1) and offsets2.shape == (H, C2 + 1)
    m1 = np.empty((B, H, (C1 + 31) // 32), np.uint32)
    m2 = np.empty((B, H, (C2 + 31) // 32), np.uint32)
    ranges = np.zeros((B, H, C2, 2), np.int32)
    n_ranges = np.empty((B, H), np.int32)
    n_keys = np.empty((B, H), np.int32)
    stats = np.empty((B, H, 4), np.float32)
    logits2 = np.empty((B, H, C2), np.float32) if want_logits2 else None
    lib().oracle_hier_select(B, H, C1, C2, d, C.c_float(sm_scale), _p(q), _p(centroids1), _p(sizes1),
                             _p(child_offsets), _p(thresh1), _p(centroids2), _p(sizes2), _p(offsets2), _p(thresh2),
                             _p(m1), _p(m2), _p(ranges), _p(n_ranges), _p(n_keys), _p(logits2), _p(stats))
    out = dict(mask1=m1, mask2=m2, ranges=ranges, n_ranges=n_ranges, n_keys=n_keys, stats=stats)
    if want_logits2:
        out["logits2"] = logits2
    return out


def hier_select_mean(q, centroids1, sizes1, child_offsets, thresh1, centroids2, sizes2, offsets2, thresh2, sm_scale):
    """Two-level lookup with the prefill rule (Appendix D: scores averaged over the Lq query tokens) at both levels
    (Section 3.3): level 1 keeps coarse clusters by their averaged Eq. 2 scores; level 2 scores the children of the
    kept coarse clusters per token with the normaliser over those children only (Eq. 3), averages over the tokens and
    keeps by T2.  Composed from centroid_score and select_mean, the candidates' arrays being cut out per (b, h).
    q [B,H,Lq,d] -> dict(mask1 [B,H,C1] bool, mask2 [B,H,C2] bool, ranges [B,H,C2,2], n_ranges, n_keys [B,H])."""
    q = _f16(q)
    B, H, Lq, d = q.shape
    centroids1, centroids2 = _f16(centroids1), _f16(centroids2)
    sizes1, child_offsets, sizes2, offsets2 = _i32(sizes1), _i32(child_offsets), _i32(sizes2), _i32(offsets2)
    thresh1, thresh2 = _f32(thresh1), _f32(thresh2)
    C1, C2 = centroids1.shape[1], centroids2.shape[1]
    x1, m1, D1 = centroid_score(q, centroids1, sizes1, sm_scale)
    fan = np.diff(child_offsets, axis=1).astype(np.int32)
    # level 1: only the mask matters (clusters with no keys underneath are never kept)
    mk1 = select_mean(x1, m1, D1, thresh1, sizes1, child_offsets)[0]
    mask1 = ((mk1[..., :, None] >> np.arange(32, dtype=np.uint32)) & 1).reshape(B, H, -1)[..., :C1].astype(bool)
    mask2 = np.zeros((B, H, C2), bool)
    ranges = np.zeros((B, H, C2, 2), np.int32)
    n_ranges = np.zeros((B, H), np.int32)
    n_keys = np.zeros((B, H), np.int32)
    for b in range(B):
        for h in range(H):
            cand = np.concatenate([np.arange(child_offsets[h, j], child_offsets[h, j + 1])
                                   for j in np.flatnonzero(mask1[b, h])] + [np.zeros(0, np.int64)]).astype(np.int64)
            if len(cand) == 0:
                continue
            cc, cs = np.ascontiguousarray(centroids2[h][cand][None]), np.ascontiguousarray(sizes2[h][cand][None])
            x2, m2, D2 = centroid_score(q[b:b + 1, h:h + 1], cc, cs, sm_scale)
            co = np.zeros((1, len(cand) + 1), np.int32)
            mk2 = select_mean(x2, m2, D2, thresh2[h:h + 1], cs, co)[0]
            kept = ((mk2[0, 0][:, None] >> np.arange(32, dtype=np.uint32)) & 1).reshape(-1)[:len(cand)].astype(bool)
            ids = cand[kept]
            mask2[b, h, ids] = True
            n_ranges[b, h] = len(ids)
            ranges[b, h, :len(ids), 0] = offsets2[h, ids]
            ranges[b, h, :len(ids), 1] = sizes2[h, ids]
            n_keys[b, h] = sizes2[h, ids].sum()
    del fan
    return dict(mask1=mask1, mask2=mask2, ranges=ranges, n_ranges=n_ranges, n_keys=n_keys)


def multilevel_select(q, levels, sm_scale):
    """Lookup through n >= 1 levels of centroids, coarsest first (Section 3.3, level after level).

    q [B,H,d] f16; levels = list of dicts(centroids [H,C,d] f16, sizes [H,C] i32, child_offsets [H,C+1] i32 --
    children in the next level, or key offsets at the last level --, thresh [H] f32).
    -> dict(masks = [keep mask of every level, [B,H,ceil(C/32)] u32], ranges [B,H,C_last,2], n_ranges, n_keys [B,H]).
    """
    q = _f16(q)
    B, H, d = q.shape
    n = len(levels)
    cen = [_f16(l["centroids"]) for l in levels]
    siz = [_i32(l["sizes"]) for l in levels]
    cof = [_i32(l["child_offsets"]) for l in levels]
    thr = [_f32(l["thresh"]) for l in levels]
    Cs = np.array([c.shape[1] for c in cen], np.int32)
    for k in range(n):
        assert cen[k].shape == (H, Cs[k], d) and siz[k].shape == (H, Cs[k]) and cof[k].shape == (H, Cs[k] + 1)
    masks = [np.zeros((B, H, (int(c) + 31) // 32), np.uint32) for c in Cs]
    ranges = np.zeros((B, H, int(Cs[-1]), 2), np.int32)
    n_ranges = np.empty((B, H), np.int32)
    n_keys = np.empty((B, H), np.int32)
    vp = lambda arrs: (C.c_void_p * n)(*[a.ctypes.data for a in arrs])
    lib().oracle_multilevel_select(B, H, n, _p(Cs), d, C.c_float(sm_scale), _p(q), vp(cen), vp(siz), vp(cof), vp(thr),
                                   vp(masks), _p(ranges), _p(n_ranges), _p(n_keys))
    return dict(masks=masks, ranges=ranges, n_ranges=n_ranges, n_keys=n_keys)


def sparse_attn(q, K_fixed, V_fixed, ranges, n_ranges, K_user, V_user, sm_scale, causal_user=False, row_sel=None):
    """q [B,H,Lq,d]; ranges [B,H,Lq,cap,2]; -> out [B,H,Lq,d] f64, lse [B,H,Lq] f64.

    `row_sel` ([B,H,Lq] bool) restricts the computation to sampled rows; other rows come back NaN.
    """
    q, K_fixed, V_fixed, K_user, V_user = _f16(q), _f16(K_fixed), _f16(V_fixed), _f16(K_user), _f16(V_user)
    ranges, n_ranges = _i32(ranges), _i32(n_ranges)
    B, H, Lq, d = q.shape
    L = K_fixed.shape[1]
    U = K_user.shape[2]
    assert K_fixed.shape == (H, L, d) and V_fixed.shape == (H, L, d)
    assert K_user.shape == (B, H, U, d) and V_user.shape == (B, H, U, d)
    assert ranges.shape[:3] == (B, H, Lq) and ranges.shape[4] == 2 and n_ranges.shape == (B, H, Lq)
    cap = ranges.shape[3]
    out = np.full((B, H, Lq, d), np.nan, np.float64)
    lse = np.full((B, H, Lq), np.nan, np.float64)
    sel = None if row_sel is None else np.ascontiguousarray(row_sel, dtype=np.uint8)
    lib().oracle_sparse_attn(B, H, Lq, L, U, d, C.c_float(sm_scale), int(bool(causal_user)), cap,
                             _p(q), _p(K_fixed), _p(V_fixed), _p(ranges), _p(n_ranges), _p(K_user), _p(V_user),
                             _p(sel), _p(out), _p(lse))
    return out, lse


def scores(q, centroids, sizes, sm_scale) -> np.ndarray:
    """Cluster scores S [nq, C] of Eq. 1 for one head, from the C oracle's (x, m, D): S_i = exp(x_i-m)/D.

    Shape contract of the workload module's `score_fn`: q [nq,d], centroids [C,d], sizes [C].
    """
    x, m, D = centroid_score(np.asarray(q)[None, None], np.asarray(centroids)[None], np.asarray(sizes)[None],
                             sm_scale)
    x, m, D = x[0, 0].astype(np.float64), m[0, 0].astype(np.float64), D[0, 0].astype(np.float64)
    return np.exp(x - m[:, None]) / D[:, None]


def gqa_decode(q, centroids, sizes, offsets, thresh, K_fixed, V_fixed, K_user, V_user, sm_scale, G):
    """Decode step with grouped-query attention (appendix "Additional Longbench Evaluation": keys and values are
    shared amongst a subset of the heads, and every head selects its clusters independently).

    q [B, Hq, d] f16 with Hq = H * G; query head hq uses K/V head hq // G -- its centroids, sizes, threshold,
    fixed-context keys and the sequence's user keys [B, H, U, d].  Each (sequence, query head) is one independent
    instance of the one-level method: scores (Eq. 1), threshold rule, exact attention over its kept keys plus all
    user keys.  Written as that definition: one call of the one-level functions per query head, on the K/V head's
    arrays.  -> dict(mask [B,Hq,W] u32, n_keys [B,Hq] i32, out [B,Hq,d] f64, lse [B,Hq] f64).
    """
    q = _f16(q)
    B, Hq, d = q.shape
    H = centroids.shape[0]
    assert Hq == H * G
    Cn = centroids.shape[1]
    W = (Cn + 31) // 32
    res = dict(mask=np.zeros((B, Hq, W), np.uint32), n_keys=np.zeros((B, Hq), np.int32),
               out=np.zeros((B, Hq, d), np.float64), lse=np.zeros((B, Hq), np.float64))
    for hq in range(Hq):
        h = hq // G
        qh = np.ascontiguousarray(q[:, hq][:, None, None, :])                       # [B, 1, 1, d]
        x, m, D = centroid_score(qh, centroids[h:h + 1], sizes[h:h + 1], sm_scale)
        mask, ranges, n_r, n_k = select(x, m, D, np.asarray(thresh)[h:h + 1], sizes[h:h + 1], offsets[h:h + 1])
        out, lse = sparse_attn(qh, K_fixed[h:h + 1], V_fixed[h:h + 1], ranges, n_r,
                               np.ascontiguousarray(K_user[:, h:h + 1]), np.ascontiguousarray(V_user[:, h:h + 1]),
                               sm_scale)
        res["mask"][:, hq] = mask[:, 0, 0]
        res["n_keys"][:, hq] = n_k[:, 0, 0]
        res["out"][:, hq] = out[:, 0, 0]
        res["lse"][:, hq] = lse[:, 0, 0]
    return res


def gqa_mean_decode(q, centroids, sizes, offsets, thresh, K_fixed, V_fixed, K_user, V_user, sm_scale, G):
    """Grouped-query decode with ONE kept set per (sequence, K/V head): the aggregation the paper's appendix
    ("Additional Longbench Evaluation") leaves as future work, read as "average the scores over the group": the
    cluster scores of Eq. 1 of the G query heads that share a K/V head are averaged (the rule of Appendix D with the
    group's heads in the place of the query tokens) and compared with T; every head of the group then attends to the
    same kept keys plus the sequence's user keys.  q [B, Hq, d], Hq = H * G, head hq uses K/V head hq // G.
    -> dict(mask [B,H,W] u32, n_keys [B,H] i32, out [B,Hq,d] f64, lse [B,Hq] f64)."""
    q = _f16(q)
    B, Hq, d = q.shape
    H = centroids.shape[0]
    assert Hq == H * G
    qg = np.ascontiguousarray(q.reshape(B, H, G, d))
    x, m, D = centroid_score(qg, centroids, sizes, sm_scale)
    mask, ranges, n_r, n_k = select_mean(x, m, D, thresh, sizes, offsets)
    cap = ranges.shape[2]
    rr = np.ascontiguousarray(np.broadcast_to(ranges[:, :, None], (B, H, G, cap, 2)))
    nn = np.ascontiguousarray(np.broadcast_to(n_r[:, :, None], (B, H, G)))
    out, lse = sparse_attn(qg, K_fixed, V_fixed, rr, nn, K_user, V_user, sm_scale)
    return dict(mask=mask, n_keys=n_k, out=out.reshape(B, Hq, d), lse=lse.reshape(B, Hq))
