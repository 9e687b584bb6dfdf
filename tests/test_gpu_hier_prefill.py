"""GPU parity of the hierarchical prefill step on averaged scores (sq_hier_prefill_mean_step) against the oracle's
composition (two-level lookup with the prefill rule at both levels, then exact attention over the kept keys)."""
import numpy as np
import pytest
import torch

from gpu_util import ATTN_ATOL, ranges_from_keep, unpack_mask
from oracle import literal
from paper_2411_09688_amd import workload as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def sq():
    from paper_2411_09688_amd import binding
    binding.lib()
    return binding


def t(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def between(sorted_desc, k):
    """A threshold between the k-th and (k+1)-th largest value, moved down to a pair that is at least 1 % apart."""
    s = sorted_desc
    k = max(0, min(k, len(s) - 2))
    while k < len(s) - 2 and not s[k] > 1.01 * s[k + 1]:
        k += 1
    return np.float32(np.sqrt(s[k] * max(s[k + 1], 1e-30)))


def thresholds(w):
    """Per head, from the literal fp64 averaged scores of sequence 0: T1 keeps about coarse_keep_frac of the coarse
    clusters, T2 about keep_frac of the keys (by count of fine clusters among the candidates)."""
    T1, T2 = np.empty(w.H, np.float32), np.empty(w.H, np.float32)
    for h in range(w.H):
        S1 = literal.select_mean(w.q[0, h], w.centroids1[h], w.sizes1[h], 0.0, w.sm_scale)[1]
        live = np.sort(S1[w.sizes1[h] > 0])[::-1]
        T1[h] = between(live, int(np.ceil(w.coarse_keep_frac * w.C1)) - 1)
        S2 = literal.hier_select_mean(w.q[0, h], w.centroids1[h], w.sizes1[h], w.child_offsets[h], T1[h],
                                      w.centroids[h], w.sizes[h], 0.0, w.sm_scale)[3]
        cand = ~np.isnan(S2) & (w.sizes[h] > 0)
        s2 = np.sort(S2[cand])[::-1]
        T2[h] = between(s2, int(np.ceil(w.keep_frac * w.C)) - 1) if len(s2) > 1 else np.float32(0.0)
    return T1, T2


def run(sq, w, T1, T2, optional=True):
    sh = sq.make_shape(w.B, w.H, w.L, w.C, w.Lq, w.U, w.sm_scale, causal_user=w.causal_user)
    out = torch.full((w.B, w.H, w.Lq, w.d), 7.0, dtype=torch.float16, device=DEV)
    lse = torch.zeros(w.B, w.H, w.Lq, dtype=torch.float32, device=DEV)
    mask = torch.zeros(w.B, w.H, (w.C + 31) // 32, dtype=torch.int32, device=DEV)
    nk = torch.zeros(w.B, w.H, dtype=torch.int32, device=DEV)
    sq.sq_hier_prefill_mean_step(sh, w.C1, t(w.q), t(w.centroids1), t(w.sizes1), t(w.child_offsets), t(T1),
                                 t(w.centroids), t(w.sizes), t(w.offsets), t(T2), t(w.K_fixed), t(w.V_fixed),
                                 t(w.K_user) if w.U else None, t(w.V_user) if w.U else None, out,
                                 lse if optional else None, mask if optional else None, nk if optional else None,
                                 sq.workspace(sh, sq.SQ_CALL_HIER_PREFILL_MEAN_STEP, DEV))
    torch.cuda.synchronize()
    return out.cpu().numpy(), lse.cpu().numpy(), mask.cpu().numpy(), nk.cpu().numpy()


def compare(oracle, w, T1, T2, got, label, sample=None):
    out, lse, mask, nk = got
    ref = oracle.hier_select_mean(w.q, w.centroids1, w.sizes1, w.child_offsets, T1, w.centroids, w.sizes, w.offsets, T2,
                                  w.sm_scale)
    gk = unpack_mask(mask, w.C)
    for b in range(w.B):
        for h in range(w.H):
            if (gk[b, h] == ref["mask2"][b, h]).all():
                continue
            # a disagreement must come from a cluster next to a threshold, at either level
            k1, k2, S1, S2 = literal.hier_select_mean(w.q[b, h], w.centroids1[h], w.sizes1[h], w.child_offsets[h], T1[h],
                                                      w.centroids[h], w.sizes[h], T2[h], w.sm_scale)
            near1 = literal.near_threshold(S1, T1[h]).any()
            d2 = np.flatnonzero(gk[b, h] != ref["mask2"][b, h])
            assert near1 or literal.near_threshold(np.nan_to_num(S2[d2], nan=1.0), T2[h]).all(), (label, b, h, d2[:8])
            print(f"[near-threshold clusters {label}] b{b} h{h}: {d2[:8].tolist()} (level-1 near: {bool(near1)})")
    np.testing.assert_array_equal(nk, (gk * w.sizes[None]).sum(-1))
    # attention over the GPU's own (validated) set, the same ranges for every query token of a (b, h)
    R = (w.B, w.H, w.Lq)
    sel = np.ones(R, bool)
    if sample is not None:
        sel = np.zeros(R, bool)
        sel.ravel()[np.random.default_rng(3).choice(sel.size, size=sample, replace=False)] = True
        sel[:, :, 0] = True
        sel[:, :, -1] = True
    cap = max(1, int(gk.sum(-1).max()))
    ranges = np.zeros((w.B, w.H, cap, 2), np.int32)
    nr = np.zeros((w.B, w.H), np.int32)
    for b in range(w.B):
        for h in range(w.H):
            ranges[b, h], nr[b, h] = ranges_from_keep(gk[b, h], w.offsets[h], w.sizes[h], cap)
    rr = np.ascontiguousarray(np.broadcast_to(ranges[:, :, None], (*R, cap, 2)))
    nn = np.ascontiguousarray(np.broadcast_to(nr[:, :, None], R))
    ro, rl = oracle.sparse_attn(w.q, w.K_fixed, w.V_fixed, rr, nn, w.K_user, w.V_user, w.sm_scale,
                                causal_user=w.causal_user, row_sel=sel)
    err = np.abs(out.astype(np.float64)[sel] - ro[sel]).max()
    assert err <= ATTN_ATOL, f"{label}: attention max-abs error {err}"
    fin = np.isfinite(rl[sel])
    assert (np.isneginf(lse[sel]) == ~fin).all()
    # (logits reach 35 on the nested mixture: fp32 accumulation of 128 fp16 products of that size is good to ~1e-4 relative)
    np.testing.assert_allclose(lse[sel][fin], rl[sel][fin], atol=2e-4, rtol=1e-4)
    return gk, err


CASES = [
    dict(B=1, H=2, L=2048, C=64, C1=8, Lq=40, U=40, keep_frac=0.25, coarse_keep_frac=0.5, causal_user=True),
    dict(B=2, H=3, L=3000, C=120, C1=10, Lq=70, U=33, keep_frac=0.2, coarse_keep_frac=0.3, causal_user=True),
    dict(B=1, H=1, L=1000, C=32, C1=4, Lq=5, U=0, keep_frac=0.3, coarse_keep_frac=0.5, causal_user=False),
    dict(B=1, H=2, L=8192, C=2048, C1=64, Lq=33, U=10, keep_frac=0.1, coarse_keep_frac=0.25, causal_user=False),
    dict(B=2, H=2, L=4096, C=256, C1=16, Lq=130, U=130, keep_frac=0.125, coarse_keep_frac=0.25, causal_user=True),
]


@pytest.mark.parametrize("case", CASES)
def test_hier_prefill_mean_step_small(sq, oracle, case):
    w = wl.make_workload("hier_prefill_mean", seed=31, threads=2, **case)
    T1, T2 = thresholds(w)
    got = run(sq, w, T1, T2)
    gk, err = compare(oracle, w, T1, T2, got, f"hier-prefill-mean{case}")
    assert 0 < gk.sum() < w.B * w.H * w.C


def test_first_level_keeping_everything_is_the_one_level_step(sq, oracle):
    w = wl.make_workload("hier_prefill_mean_all", B=1, H=2, L=4096, C=128, C1=8, Lq=50, U=20, keep_frac=0.2,
                         coarse_keep_frac=0.5, causal_user=True, seed=32, threads=2)
    _, T2 = thresholds(w)
    T1 = np.full(w.H, -1.0, np.float32)
    out, lse, mask, nk = run(sq, w, T1, T2)
    sh = sq.make_shape(w.B, w.H, w.L, w.C, w.Lq, w.U, w.sm_scale, causal_user=True)
    out1 = torch.empty(w.B, w.H, w.Lq, w.d, dtype=torch.float16, device=DEV)
    mask1 = torch.zeros(w.B, w.H, (w.C + 31) // 32, dtype=torch.int32, device=DEV)
    nk1 = torch.zeros(w.B, w.H, dtype=torch.int32, device=DEV)
    sq.sq_prefill_mean_step(sh, t(w.q), t(w.centroids), t(w.sizes), t(w.offsets), t(T2), t(w.K_fixed), t(w.V_fixed),
                            t(w.K_user), t(w.V_user), out1, None, mask1, nk1,
                            sq.workspace(sh, sq.SQ_CALL_PREFILL_MEAN_STEP, DEV))
    torch.cuda.synchronize()
    # every fine cluster is a candidate, in order: the same sums in the same order
    np.testing.assert_array_equal(mask, mask1.cpu().numpy())
    np.testing.assert_array_equal(nk, nk1.cpu().numpy())
    np.testing.assert_array_equal(out, out1.cpu().numpy())


def test_nothing_kept_and_optional_outputs(sq, oracle):
    w = wl.make_workload("hier_prefill_mean_none", B=1, H=2, L=2048, C=64, C1=8, Lq=20, U=16, keep_frac=0.25,
                         coarse_keep_frac=0.5, causal_user=True, seed=33, threads=2)
    T1, T2 = thresholds(w)
    big = np.full(w.H, 10.0, np.float32)
    for a, b in ((big, T2), (T1, big)):                          # no coarse cluster kept / no fine cluster kept
        out, lse, mask, nk = run(sq, w, a, b)
        assert nk.sum() == 0 and not mask.any()
        compare(oracle, w, a, b, (out, lse, mask, nk), "nothing kept")    # attention over the user keys alone
    ref = run(sq, w, T1, T2)
    got = run(sq, w, T1, T2, optional=False)
    np.testing.assert_array_equal(got[0], ref[0])


def test_hier_prefill_mean_long_context_shape(sq, oracle):
    """A slice of the long-context config's hierarchy (256 coarse -> 16384 fine clusters) with a 256-token input."""
    print("hier prefill mean: generating", flush=True)
    w = wl.make_workload("hier_prefill_mean_big", B=1, H=2, L=262144, C=16384, C1=256, Lq=256, U=256, keep_frac=1 / 16,
                         coarse_keep_frac=1 / 8, causal_user=True, seed=34, threads=8)
    T1, T2 = thresholds(w)
    got = run(sq, w, T1, T2)
    gk, err = compare(oracle, w, T1, T2, got, "hier-prefill-mean-big")
    print("hier prefill mean attention max-abs err", err, "keep", got[3].mean() / w.L, flush=True)
    assert 0 < gk.sum()


# ---- per-query selection through the hierarchy (sq_hier_prefill_step) -----------------------------------------------

def run_per_query(sq, w, T1, T2, optional=True):
    sh = sq.make_shape(w.B, w.H, w.L, w.C, w.Lq, w.U, w.sm_scale, causal_user=w.causal_user)
    out = torch.full((w.B, w.H, w.Lq, w.d), 7.0, dtype=torch.float16, device=DEV)
    lse = torch.zeros(w.B, w.H, w.Lq, dtype=torch.float32, device=DEV)
    mask = torch.zeros(w.B, w.H, w.Lq, (w.C + 31) // 32, dtype=torch.int32, device=DEV)
    nk = torch.zeros(w.B, w.H, w.Lq, dtype=torch.int32, device=DEV)
    sq.sq_hier_prefill_step(sh, w.C1, t(w.q), t(w.centroids1), t(w.sizes1), t(w.child_offsets), t(T1), t(w.centroids),
                            t(w.sizes), t(w.offsets), t(T2), t(w.K_fixed), t(w.V_fixed),
                            t(w.K_user) if w.U else None, t(w.V_user) if w.U else None, out,
                            lse if optional else None, mask if optional else None, nk if optional else None,
                            sq.workspace(sh, sq.SQ_CALL_HIER_PREFILL_STEP, DEV))
    torch.cuda.synchronize()
    return out.cpu().numpy(), lse.cpu().numpy(), mask.cpu().numpy(), nk.cpu().numpy()


def per_query_thresholds(w):
    """Per head, from the literal scores of the first token of sequence 0 (Eq. 2, then Eq. 3 over its candidates)."""
    T1, T2 = np.empty(w.H, np.float32), np.empty(w.H, np.float32)
    for h in range(w.H):
        S1 = literal.scores(w.q[0, h, :1], w.centroids1[h], w.sizes1[h], w.sm_scale)[0]
        T1[h] = between(np.sort(S1[w.sizes1[h] > 0])[::-1], int(np.ceil(w.coarse_keep_frac * w.C1)) - 1)
        S2 = literal.hier_select(w.q[0, h, 0], w.centroids1[h], w.sizes1[h], w.child_offsets[h], T1[h], w.centroids[h],
                                 w.sizes[h], 0.0, w.sm_scale)[3]
        s2 = np.sort(S2[~np.isnan(S2) & (w.sizes[h] > 0)])[::-1]
        T2[h] = between(s2, int(np.ceil(w.keep_frac * w.C)) - 1) if len(s2) > 1 else np.float32(0.0)
    return T1, T2


def compare_per_query(oracle, w, T1, T2, got, label, sample=None):
    out, lse, mask, nk = got
    B, H, Lq, C = w.B, w.H, w.Lq, w.C
    gk = unpack_mask(mask, C)                                    # [B, H, Lq, C]
    listed = 0
    for b in range(B):
        # the decode-time two-level oracle with the Lq tokens of a sequence in the place of a batch
        qb = np.ascontiguousarray(w.q[b].transpose(1, 0, 2))     # [Lq, H, d]
        ref = oracle.hier_select(qb, w.centroids1, w.sizes1, w.child_offsets, T1, w.centroids, w.sizes, w.offsets, T2,
                                 w.sm_scale)
        ok = unpack_mask(ref["mask2"], C)                        # [Lq, H, C]
        for tkn, h in np.argwhere((gk[b].transpose(1, 0, 2) != ok).any(-1)):
            k1, k2, S1, S2 = literal.hier_select(w.q[b, h, tkn], w.centroids1[h], w.sizes1[h], w.child_offsets[h], T1[h],
                                                 w.centroids[h], w.sizes[h], T2[h], w.sm_scale)
            d2 = np.flatnonzero(gk[b, h, tkn] != ok[tkn, h])
            near1 = literal.near_threshold(S1, T1[h]).any()
            assert near1 or literal.near_threshold(np.nan_to_num(S2[d2], nan=1.0), T2[h]).all(), (label, b, h, tkn, d2[:8])
            listed += 1
    if listed:
        print(f"[{label}] {listed} (token, head) rows with a near-threshold cluster decided differently")
    np.testing.assert_array_equal(nk, (gk * w.sizes[None, :, None, :]).sum(-1))
    # attention over the GPU's own (validated) per-token sets
    R = (B, H, Lq)
    sel = np.ones(R, bool)
    if sample is not None:
        sel = np.zeros(R, bool)
        sel.ravel()[np.random.default_rng(4).choice(sel.size, size=sample, replace=False)] = True
        sel[:, :, 0] = True
        sel[:, :, -1] = True
    cap = max(1, int(gk.sum(-1).max()))
    ranges = np.zeros((*R, cap, 2), np.int32)
    nr = np.zeros(R, np.int32)
    for b, h, tkn in np.argwhere(sel):
        ranges[b, h, tkn], nr[b, h, tkn] = ranges_from_keep(gk[b, h, tkn], w.offsets[h], w.sizes[h], cap)
    ro, rl = oracle.sparse_attn(w.q, w.K_fixed, w.V_fixed, ranges, nr, w.K_user, w.V_user, w.sm_scale,
                                causal_user=w.causal_user, row_sel=sel)
    err = np.abs(out.astype(np.float64)[sel] - ro[sel]).max()
    assert err <= ATTN_ATOL, f"{label}: attention max-abs error {err}"
    fin = np.isfinite(rl[sel])
    assert (np.isneginf(lse[sel]) == ~fin).all()
    np.testing.assert_allclose(lse[sel][fin], rl[sel][fin], atol=2e-4, rtol=1e-4)
    return gk, err


@pytest.mark.parametrize("case", CASES[:3] + [CASES[4]])
def test_hier_prefill_step_small(sq, oracle, case):
    w = wl.make_workload("hier_prefill", seed=36, threads=2, **case)
    T1, T2 = per_query_thresholds(w)
    got = run_per_query(sq, w, T1, T2)
    gk, err = compare_per_query(oracle, w, T1, T2, got, f"hier-prefill{case}")
    assert 0 < gk.sum() < gk.size


def test_per_query_first_level_keeping_everything_is_the_one_level_step(sq, oracle):
    w = wl.make_workload("hier_prefill_all", B=1, H=2, L=4096, C=128, C1=8, Lq=50, U=20, keep_frac=0.2,
                         coarse_keep_frac=0.5, causal_user=True, seed=37, threads=2)
    _, T2 = per_query_thresholds(w)
    out, lse, mask, nk = run_per_query(sq, w, np.full(w.H, -1.0, np.float32), T2)
    sh = sq.make_shape(w.B, w.H, w.L, w.C, w.Lq, w.U, w.sm_scale, causal_user=True)
    out1 = torch.empty(w.B, w.H, w.Lq, w.d, dtype=torch.float16, device=DEV)
    mask1 = torch.zeros(w.B, w.H, w.Lq, (w.C + 31) // 32, dtype=torch.int32, device=DEV)
    nk1 = torch.zeros(w.B, w.H, w.Lq, dtype=torch.int32, device=DEV)
    sq.sq_prefill_step(sh, t(w.q), t(w.centroids), t(w.sizes), t(w.offsets), t(T2), t(w.K_fixed), t(w.V_fixed),
                       t(w.K_user), t(w.V_user), out1, None, mask1, nk1, sq.workspace(sh, sq.SQ_CALL_PREFILL_STEP, DEV))
    torch.cuda.synchronize()
    np.testing.assert_array_equal(mask, mask1.cpu().numpy())     # every fine cluster is a candidate of every token
    np.testing.assert_array_equal(nk, nk1.cpu().numpy())
    np.testing.assert_array_equal(out, out1.cpu().numpy())
    assert nk.sum() > 0


def test_per_query_more_than_1024_coarse_clusters_is_refused(sq):
    sh = sq.make_shape(1, 1, 4096, 2048, 4, 0, 0.1)
    z = torch.zeros(64, dtype=torch.float16, device=DEV)
    zi = torch.zeros(64, dtype=torch.int32, device=DEV)
    zf = torch.zeros(64, dtype=torch.float32, device=DEV)
    with pytest.raises(sq.SqError) as e:
        sq.sq_hier_prefill_step(sh, 1500, z, z, zi, zi, zf, z, zi, zi, zf, z, z, None, None, z, None, None, None,
                                sq.workspace(sh, sq.SQ_CALL_HIER_PREFILL_STEP, DEV))
    assert e.value.code == sq.SQ_ERR_UNSUPPORTED
