"""Seeded synthetic workloads shaped like the paper's long-context runs.

The paper benchmarks its kernels on K/V produced by 7B LLaMA-family models
(H=32, d=128) over language-modelling text with K-means centroids (Appendix
"Kernel Benchmarking").  Neither the text, the weights nor the authors'
clustering is available, so Gaussian mixtures with the same shapes stand in:
per head, `C` cluster centres ~ N(0, I_d), cluster sizes ~ Multinomial(L,
uniform), key = centre + noise * N(0, I_d), keys stored sorted by cluster id,
centroid = exact mean of the cluster's fp16 keys (Section 3.1: a centroid is
the mean of the vectors in the cluster).

This module only draws random numbers, sorts, and averages keys into
centroids.  It contains none of the online method's arithmetic: cluster
scores are always obtained through a `score_fn` the caller passes in, so the
same generator can feed the CPU oracle and the GPU library without either
side leaning on the other.
"""
from __future__ import annotations

import math
import zlib
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Callable, Optional

import numpy as np

F16 = np.float16
NOISE = 0.3            # within-cluster key / query noise of the configs
COARSE_NOISE = 1.0     # fine-centre spread around a coarse centre (two-level config)
N_CALIB = 32           # calibration queries per head


def _rng(seed: int, cfg: str, tensor: str, head: int = 0) -> np.random.Generator:
    """Independent sub-stream keyed by (seed, config, tensor name, head)."""
    key = [seed, zlib.crc32(cfg.encode()), zlib.crc32(tensor.encode()), head]
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence(key)))


def _normal(rng, shape) -> np.ndarray:
    return rng.standard_normal(shape, dtype=np.float32)


@dataclass
class Workload:
    name: str
    B: int
    H: int
    d: int
    L: int
    C: int
    Lq: int
    U: int
    sm_scale: float
    causal_user: bool
    keep_frac: float
    seed: int
    K_fixed: np.ndarray            # [H, L, d] f16, sorted by cluster id
    V_fixed: np.ndarray            # [H, L, d] f16
    centroids: np.ndarray          # [H, C, d] f16 (fine level when hierarchical)
    sizes: np.ndarray              # [H, C] i32
    offsets: np.ndarray            # [H, C+1] i32, exclusive prefix sum of sizes
    q: np.ndarray                  # [B, H, Lq, d] f16
    K_user: np.ndarray             # [B, H, U, d] f16
    V_user: np.ndarray             # [B, H, U, d] f16
    q_calib: np.ndarray            # [H, N_CALIB, d] f16
    # two-level hierarchy (C1 == 0 when absent)
    C1: int = 0
    coarse_keep_frac: float = 0.0
    centroids1: Optional[np.ndarray] = None     # [H, C1, d] f16
    sizes1: Optional[np.ndarray] = None         # [H, C1] i32, keys under each coarse cluster
    child_offsets: Optional[np.ndarray] = None  # [H, C1+1] i32 into the fine clusters
    thresh: Optional[np.ndarray] = None         # [H] f32, set by calibrate()
    thresh1: Optional[np.ndarray] = None        # [H] f32 (hierarchical)
    thresh2: Optional[np.ndarray] = None        # [H] f32 (hierarchical)
    extra: dict = field(default_factory=dict)


def _cluster_means(keys16: np.ndarray, sizes: np.ndarray, centres: np.ndarray) -> np.ndarray:
    """Exact per-cluster mean of the fp16 keys, accumulated in fp64, rounded to fp16.

    Empty clusters (size 0) keep their generating centre as a placeholder; they
    hold no keys, so the value is never meaningful.
    """
    C, d = centres.shape
    out = centres.astype(np.float64)
    nz = np.flatnonzero(sizes > 0)
    starts = np.concatenate([[0], np.cumsum(sizes)[:-1]])[nz]
    step = 1 << 16
    sums = np.zeros((len(nz), d), dtype=np.float64)
    # reduceat over non-empty segments only (consecutive non-empty starts are strictly increasing)
    L = keys16.shape[0]
    if L <= step * 4:
        sums = np.add.reduceat(keys16.astype(np.float64), starts, axis=0)
    else:
        # chunked to bound the fp64 temporary: split at cluster boundaries
        bounds = np.concatenate([starts, [L]])
        i = 0
        while i < len(nz):
            j = int(np.searchsorted(bounds, bounds[i] + step, side="right")) - 1
            j = max(j, i + 1)
            j = min(j, len(nz))
            seg = keys16[bounds[i]:bounds[j]].astype(np.float64)
            sums[i:j] = np.add.reduceat(seg, bounds[i:j] - bounds[i], axis=0)
            i = j
    out[nz] = sums / sizes[nz, None]
    return out.astype(F16)


def _head_fixed(seed, cfg, h, L, C, d, centres=None, scale=1.0):
    """One head of the fixed context: centres, sizes, sorted keys, values, centroids."""
    if centres is None:
        centres = np.float32(scale) * _normal(_rng(seed, cfg, "centres", h), (C, d))
    sizes = _rng(seed, cfg, "sizes", h).multinomial(L, np.full(C, 1.0 / C)).astype(np.int32)
    ids = np.repeat(np.arange(C, dtype=np.int32), sizes)
    rk = _rng(seed, cfg, "K_fixed", h)
    K = np.empty((L, d), dtype=F16)
    step = 1 << 16
    for s in range(0, L, step):
        e = min(L, s + step)
        K[s:e] = (centres[ids[s:e]] + NOISE * _normal(rk, (e - s, d))).astype(F16)
    rv = _rng(seed, cfg, "V_fixed", h)
    V = np.empty((L, d), dtype=F16)
    for s in range(0, L, step):
        e = min(L, s + step)
        V[s:e] = _normal(rv, (e - s, d)).astype(F16)
    cent = _cluster_means(K, sizes, centres)
    return centres, sizes, K, V, cent


def _queries(seed, cfg, tensor, h, n, centres):
    r = _rng(seed, cfg, tensor, h)
    pick = r.integers(0, centres.shape[0], size=n)
    return (centres[pick] + NOISE * _normal(r, (n, centres.shape[1]))).astype(F16)


def make_workload(name: str, *, B: int, H: int, L: int, C: int, Lq: int, U: int,
                  keep_frac: float, d: int = 128, seed: int = 0, causal_user: bool = False,
                  C1: int = 0, coarse_keep_frac: float = 0.0, threads: int = 8, head_skew: float = 0.0,
                  variable_fanout: bool = False) -> Workload:
    """Draw one workload.  `C1 > 0` makes the nested two-level mixture (C % C1 == 0).

    `head_skew` > 0 (one-level only) makes the heads differ in how peaked their score distributions are, as the
    heads of a model do (appendix "Attention Score Skewness"): head h draws its centres with standard deviation
    1 + head_skew * (2 h / (H - 1) - 1), so low heads spread their estimated attention over many clusters and high
    heads concentrate it on one.  Under ONE threshold for all heads (Section 3.2) the heads then keep very different
    numbers of keys -- the imbalance the split-KV scheme of Section 4.2 exists for.

    `variable_fanout` (two-level): every coarse cluster gets one fine cluster plus a multinomial share of the other
    C - C1, so the fan-out varies from cluster to cluster and C need not be a multiple of C1 -- what clustering the
    fine centroids produces (Section 3.3), e.g. the paper's sizing of fine centroids at 5 % and coarse centroids at
    1 % or 0.5 % of the context length (Section 6, "Experimental Details")."""
    if C1:
        assert (variable_fanout or C % C1 == 0) and head_skew == 0.0 and C >= C1
    fan = C // C1 if C1 else 0

    def one_head(h):
        centres_fine = None
        if C1:
            coarse = _normal(_rng(seed, name, "coarse_centres", h), (C1, d))
            if variable_fanout:
                fans = 1 + _rng(seed, name, "fanout", h).multinomial(C - C1, np.full(C1, 1.0 / C1))
            else:
                fans = np.full(C1, fan)
            co = np.concatenate([[0], np.cumsum(fans)]).astype(np.int32)
            centres_fine = (np.repeat(coarse, fans, axis=0)
                            + COARSE_NOISE * _normal(_rng(seed, name, "centres", h), (C, d)))
        scale = 1.0 + head_skew * (2.0 * h / max(1, H - 1) - 1.0)
        centres, sizes, K, V, cent = _head_fixed(seed, name, h, L, C, d, centres_fine, scale)
        qs = _queries(seed, name, "q", h, B * Lq, centres).reshape(B, Lq, d)
        qc = _queries(seed, name, "q_calib", h, N_CALIB, centres)
        ru = _rng(seed, name, "user", h)
        Ku = _normal(ru, (B, U, d)).astype(F16)
        Vu = _normal(ru, (B, U, d)).astype(F16)
        res = dict(sizes=sizes, K=K, V=V, cent=cent, q=qs, qc=qc, Ku=Ku, Vu=Vu)
        if C1:
            # Level-1 centroid = unweighted mean of its child level-2 centroids (K-means run on
            # the level-2 centroids, Section 3.3); level-1 size = number of keys underneath.
            c1 = (np.add.reduceat(cent.astype(np.float64), co[:-1], axis=0) / fans[:, None]).astype(F16)
            res["cent1"] = c1
            res["sizes1"] = np.add.reduceat(sizes.astype(np.int64), co[:-1]).astype(np.int32)
            res["co"] = co
        return res

    with ThreadPoolExecutor(max_workers=max(1, threads)) as ex:
        heads = list(ex.map(one_head, range(H)))

    sizes = np.stack([r["sizes"] for r in heads])
    offsets = np.zeros((H, C + 1), dtype=np.int32)
    offsets[:, 1:] = np.cumsum(sizes, axis=1)
    w = Workload(
        name=name, B=B, H=H, d=d, L=L, C=C, Lq=Lq, U=U,
        sm_scale=float(np.float32(1.0 / math.sqrt(d))), causal_user=causal_user,
        keep_frac=keep_frac, seed=seed,
        K_fixed=np.stack([r["K"] for r in heads]), V_fixed=np.stack([r["V"] for r in heads]),
        centroids=np.stack([r["cent"] for r in heads]), sizes=sizes, offsets=offsets,
        q=np.ascontiguousarray(np.stack([r["q"] for r in heads], axis=1)),
        K_user=np.ascontiguousarray(np.stack([r["Ku"] for r in heads], axis=1)),
        V_user=np.ascontiguousarray(np.stack([r["Vu"] for r in heads], axis=1)),
        q_calib=np.stack([r["qc"] for r in heads]),
    )
    if C1:
        w.C1 = C1
        w.coarse_keep_frac = coarse_keep_frac
        w.centroids1 = np.stack([r["cent1"] for r in heads])
        w.sizes1 = np.stack([r["sizes1"] for r in heads])
        w.child_offsets = np.stack([r["co"] for r in heads])
    return w


# The five benchmark configurations (shapes from the benchmark's config list; d=128, fp16, seed 0).
CONFIGS = {
    "cfg1_tiny_decode": dict(B=1, H=4, L=4096, C=64, Lq=1, U=128, keep_frac=1 / 4),
    "cfg2_decode_32k": dict(B=1, H=32, L=32768, C=1024, Lq=1, U=512, keep_frac=1 / 8),
    "cfg3_batched_decode_32k": dict(B=16, H=32, L=32768, C=1024, Lq=1, U=256, keep_frac=1 / 8),
    "cfg4_prefill_32k": dict(B=1, H=32, L=32768, C=1024, Lq=1024, U=1024, keep_frac=1 / 8,
                             causal_user=True),
    "cfg5_hier_decode_512k": dict(B=1, H=32, L=524288, C=16384, Lq=1, U=1024, keep_frac=1 / 16,
                                  C1=256, coarse_keep_frac=1 / 8),
}

# The paper's own sizing of the two-level hierarchy (Section 6 "Experimental Details"; appendix "Hierarchical kernel
# benchmarking"): fine centroids at 5 % of the context length, coarse centroids at 1 % (or 0.5 %), the first level
# pruning 50 % (or 90 %) of the coarse clusters, variable fan-out.  256K keys: 5 % of the 512K context of config 5
# would be more fine clusters per head than the lookup kernels take (16384).
HIER_SIZING_CONFIGS = {
    "f3_hier_1pct_prune50_256k": dict(B=1, H=32, L=262144, C=13107, Lq=1, U=1024, keep_frac=1 / 10, C1=2621,
                                      coarse_keep_frac=0.5, variable_fanout=True),
    "f3_hier_05pct_prune90_256k": dict(B=1, H=32, L=262144, C=13107, Lq=1, U=1024, keep_frac=1 / 10, C1=1310,
                                       coarse_keep_frac=0.1, variable_fanout=True),
}

# Grouped-query decode at a Llama-3.1-8B attention shape (32 query heads over 8 K/V heads, 32K fixed context): not
# one of the five configurations above; the "next" row for models whose heads share keys and values.  Lq holds
# the group size G: the G query heads of a K/V head are its G query rows, q [B, H, G, d] = q [B, H*G, 1, d].
GQA_CONFIGS = {
    "gqa_decode_32k": dict(B=1, H=8, L=32768, C=1024, Lq=4, U=512, keep_frac=1 / 8),
}


# Offline clustering of the headline config's fixed context: 32 heads x 32768 keys into 1024 clusters (Section 3.1).
KMEANS_CONFIGS = {
    "kmeans_32k": dict(H=32, L=32768, C=1024),
}


def make_config(name: str, seed: int = 0, threads: int = 8, **override) -> Workload:
    kw = dict(CONFIGS[name] if name in CONFIGS else HIER_SIZING_CONFIGS[name] if name in HIER_SIZING_CONFIGS
              else GQA_CONFIGS[name])
    kw.update(override)
    return make_workload(name, seed=seed, threads=threads, **kw)


def extra_queries(w: Workload, n: int, tensor: str = "q_bench") -> np.ndarray:
    """`n` further decode queries per head, [n, H, d] f16, drawn like `w.q` (centroid + noise).

    The generating centres are not kept, so the (fp16) centroids stand in for them; at cluster
    sizes of ~32 keys the centroid is within noise/sqrt(32) of the centre.
    """
    out = np.empty((n, w.H, w.d), dtype=F16)
    for h in range(w.H):
        out[:, h] = _queries(w.seed, w.name, tensor, h, n, w.centroids[h].astype(np.float32))
    return out


def clustering_input(seed: int, H: int, L: int, C: int, d: int = 128, mix: int = 0, name: str = "kmeans"):
    """Input of the offline clustering step: UNSORTED keys and values of a fixed context plus a seeding.

    Keys are the mixture of the configs (centre + NOISE * N(0, I), `mix` generating centres, default C) in random
    token order, as a real context delivers them.  The seeding is the usual "C distinct keys drawn at random":
    `init` holds their indices, so each side normalises them itself.
    -> K [H, L, d] f16, V [H, L, d] f16, init [H, C] int32."""
    mix = mix or C
    K = np.empty((H, L, d), dtype=F16)
    V = np.empty((H, L, d), dtype=F16)
    init = np.empty((H, C), dtype=np.int32)
    for h in range(H):
        centres = _normal(_rng(seed, name, "centres", h), (mix, d))
        r = _rng(seed, name, "K", h)
        ids = r.integers(0, mix, size=L)
        K[h] = (centres[ids] + NOISE * _normal(r, (L, d))).astype(F16)
        V[h] = _normal(_rng(seed, name, "V", h), (L, d)).astype(F16)
        init[h] = np.sort(_rng(seed, name, "init", h).choice(L, size=C, replace=False)).astype(np.int32)
    return K, V, init


# --------------------------------------------------------------------------------------------
# Threshold calibration.  `score_fn(q[nq,d] f16, centroids[C,d] f16, sizes[C] i32, sm_scale)`
# returns the cluster scores S[nq, C] of Eq. 1 and is supplied by the caller.
# --------------------------------------------------------------------------------------------
ScoreFn = Callable[[np.ndarray, np.ndarray, np.ndarray, float], np.ndarray]


def _cut(scores: np.ndarray, weights: np.ndarray, target: float) -> float:
    """Threshold between the last score needed to reach `target` total weight and the next one."""
    order = np.argsort(-scores, kind="stable")
    s = scores[order]
    cum = np.cumsum(weights[order].astype(np.float64))
    k = int(np.searchsorted(cum, target, side="left"))      # s[0..k] kept
    k = min(k, len(s) - 1)
    lo = s[k + 1] if k + 1 < len(s) else s[k] * 0.5
    # geometric mean of last-in and first-out; strict '>' then keeps exactly s[0..k]
    return float(math.sqrt(float(s[k]) * float(max(lo, 1e-300))))


def calibrate(w: Workload, score_fn: ScoreFn, global_threshold: bool = False) -> Workload:
    """Per-head thresholds from the calibration queries, to hit the configured key fraction.

    `global_threshold` (one-level): ONE threshold for all heads, as in Section 3.2 / Appendix C -- the (S_i, N_i) of
    every head's calibration queries are pooled and the cut keeps keep_frac of all pooled keys; every head gets that
    value, and heads whose scores are flatter keep more keys than heads whose scores are peaked.

    One-level: pool (S_i, N_i) over the calibration queries, keep the highest scores until
    keep_frac of the pooled keys is covered.  Two-level: T1 keeps coarse_keep_frac of the coarse
    clusters (by count); T2, applied to the children of the kept coarse clusters with the
    normaliser over those children only (Section 3.3), keeps keep_frac of the keys overall.
    """
    H = w.H
    if not w.C1:
        T = np.empty(H, dtype=np.float32)
        pooled_s, pooled_w = [], []
        for h in range(H):
            S = np.asarray(score_fn(w.q_calib[h], w.centroids[h], w.sizes[h], w.sm_scale), dtype=np.float64)
            wts = np.broadcast_to(w.sizes[h], S.shape)
            if global_threshold:
                pooled_s.append(S.ravel())
                pooled_w.append(wts.ravel())
            else:
                T[h] = _cut(S.ravel(), wts.ravel(), w.keep_frac * N_CALIB * w.L)
        if global_threshold:
            T[:] = _cut(np.concatenate(pooled_s), np.concatenate(pooled_w), w.keep_frac * N_CALIB * w.L * H)
        w.thresh = T
        return w
    T1 = np.empty(H, dtype=np.float32)
    T2 = np.empty(H, dtype=np.float32)
    for h in range(H):
        S1 = np.asarray(score_fn(w.q_calib[h], w.centroids1[h], w.sizes1[h], w.sm_scale), dtype=np.float64)
        T1[h] = _cut(S1.ravel(), np.ones(S1.size), w.coarse_keep_frac * S1.size)
        pooled_s, pooled_n = [], []
        co = w.child_offsets[h]
        for i in range(N_CALIB):
            kept = np.flatnonzero((S1[i] > np.float64(T1[h])) & (w.sizes1[h] > 0))
            cand = np.concatenate([np.arange(co[j], co[j + 1]) for j in kept]) if len(kept) else np.zeros(0, int)
            if len(cand) == 0:
                continue
            S2 = np.asarray(score_fn(w.q_calib[h, i:i + 1], w.centroids[h][cand], w.sizes[h][cand], w.sm_scale),
                            dtype=np.float64)[0]
            pooled_s.append(S2)
            pooled_n.append(w.sizes[h][cand])
        T2[h] = _cut(np.concatenate(pooled_s), np.concatenate(pooled_n), w.keep_frac * N_CALIB * w.L)
    w.thresh1, w.thresh2 = T1, T2
    return w
