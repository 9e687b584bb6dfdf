"""Helpers of the GPU parity tests: run the oracle on a host workload, run the C-ABI library on the
same arrays, and compare under the stated tolerances."""
import numpy as np
import torch

from oracle import literal

# Tolerances (the test bar):
#   selections  bit-exact, except clusters whose literal fp64 score lies within 1e-5 of T in the log
#               domain, which are listed;
#   attention   max-abs error 2e-3 on the fp16 output;
#   logits      two fp32 evaluations of a 128-term dot product of magnitude <~ 16 in different
#               summation orders differ by a few ulp of the partial sums: 2e-5 absolute is >10x that;
#   denom       relative 2e-5 (sum of C positive fp32 terms in a different order + exp ulp).
ATTN_ATOL = 2e-3
LOGIT_ATOL = 2e-5
DENOM_RTOL = 2e-5


def unpack_mask(mask, C):
    m = np.asarray(mask).view(np.uint32)
    bits = (m[..., :, None] >> np.arange(32, dtype=np.uint32)) & 1
    return bits.reshape(*m.shape[:-1], -1)[..., :C].astype(bool)


def oracle_one_level(o, w, thresh=None):
    th = w.thresh if thresh is None else thresh
    x, m, D = o.centroid_score(w.q, w.centroids, w.sizes, w.sm_scale)
    mask, ranges, nr, nk = o.select(x, m, D, th, w.sizes, w.offsets)
    return dict(logits=x, row_max=m, denom=D, mask=mask, ranges=ranges, n_ranges=nr, n_keys=nk)


def ranges_from_keep(keep_row, offsets_h, sizes_h, cap):
    ids = np.flatnonzero(keep_row)
    r = np.zeros((cap, 2), np.int32)
    r[:len(ids), 0] = offsets_h[ids]
    r[:len(ids), 1] = sizes_h[ids]
    return r, len(ids)


def check_selection(w, gpu_keep, ora_keep, thresh, centroids=None, sizes=None, label=""):
    """gpu_keep / ora_keep: bool [B,H,Lq,C].  Every disagreement must sit next to the threshold."""
    centroids = w.centroids if centroids is None else centroids
    sizes = w.sizes if sizes is None else sizes
    diff = gpu_keep != ora_keep
    listed = []
    for b, h, t, c in np.argwhere(diff):
        S = literal.scores(w.q[b, h, t:t + 1], centroids[h], sizes[h], w.sm_scale)[0]
        assert literal.near_threshold(S[c], thresh[h]), (
            f"{label} cluster {(b, h, t, c)}: gpu={gpu_keep[b, h, t, c]} oracle={ora_keep[b, h, t, c]} "
            f"S={S[c]:.9e} T={thresh[h]:.9e} (outside the near-threshold band)")
        listed.append((int(b), int(h), int(t), int(c), float(S[c]), float(thresh[h])))
    if listed:
        print(f"[near-threshold clusters {label}] " + "; ".join(
            f"(b{b},h{h},t{t},c{c}) S={s:.7e} T={T:.7e}" for b, h, t, c, s, T in listed))
    return listed


def expand_ranges(ranges, n):
    out = []
    for s, l in np.asarray(ranges)[:n]:
        out.extend(range(int(s), int(s + l)))
    return out


def dev(a, device="cuda:0"):
    return torch.from_numpy(np.ascontiguousarray(a)).to(device)
