"""GPU parity: prefill with per-query selection (scores -> masks -> sq_sparse_attn_prefill) against the oracle."""
import numpy as np
import pytest
import torch

from gpu_util import ATTN_ATOL, LOGIT_ATOL, check_selection, dev, ranges_from_keep, unpack_mask
from paper_2411_09688_amd import workload as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sq():
    from paper_2411_09688_amd import binding
    binding.lib()
    return binding


def run_prefill(sq, w, P):
    sh = P.shape
    sq.sq_centroid_score(sh, P.q, P.centroids, P.sizes, P.logits, P.row_max, P.denom)
    sq.sq_select(sh, P.logits, P.row_max, P.denom, P.thresh, P.sizes, P.offsets, P.keep_mask, None, P.n_ranges,
                 P.n_keys)
    ws = sq.workspace(sh, sq.SQ_CALL_ATTN_PREFILL, P.q.device)
    sq.sq_sparse_attn_prefill(sh, P.q, P.K_fixed, P.V_fixed, P.offsets, P.keep_mask, P.K_user, P.V_user, P.out, P.lse,
                              ws)
    torch.cuda.synchronize()


def compare_prefill(oracle, w, P, label, sample=None, rng=None, logits=True):
    """Selection of every row against the oracle; attention on all rows or on `sample` random rows."""
    C = w.C
    x, m, D = oracle.centroid_score(w.q, w.centroids, w.sizes, w.sm_scale)
    mask, _, nr, nk = oracle.select(x, m, D, w.thresh, w.sizes, w.offsets)
    if logits:
        np.testing.assert_allclose(P.logits.cpu().numpy(), x, atol=LOGIT_ATOL, rtol=0)
    gk = unpack_mask(P.keep_mask.cpu().numpy(), C)
    check_selection(w, gk, unpack_mask(mask, C), w.thresh, label=label)
    np.testing.assert_array_equal(P.n_keys.cpu().numpy(), (gk * w.sizes[None, :, None, :]).sum(-1))
    R = (w.B, w.H, w.Lq)
    sel = np.ones(R, bool)
    if sample is not None:
        sel = np.zeros(R, bool)
        idx = rng.choice(sel.size, size=sample, replace=False)
        sel.ravel()[idx] = True
        sel[:, :, 0] = True; sel[:, :, -1] = True          # causal boundary rows of every head
    cap = int(gk.sum(-1)[sel].max()) + 1
    ranges = np.zeros((*R, cap, 2), np.int32); n_r = np.zeros(R, np.int32)
    for b, h, t in np.argwhere(sel):
        ranges[b, h, t], n_r[b, h, t] = ranges_from_keep(gk[b, h, t], w.offsets[h], w.sizes[h], cap)
    out, lse = oracle.sparse_attn(w.q, w.K_fixed, w.V_fixed, ranges, n_r, w.K_user, w.V_user, w.sm_scale,
                                  causal_user=w.causal_user, row_sel=sel)
    got = P.out.cpu().numpy().astype(np.float64)
    err = np.abs(got[sel] - out[sel]).max()
    assert err <= ATTN_ATOL, f"{label}: attention max-abs error {err} over {sel.sum()} rows"
    glse = P.lse.cpu().numpy()
    np.testing.assert_allclose(glse[sel], lse[sel], atol=2e-4, rtol=1e-5)
    return err


@pytest.mark.parametrize("case", [
    dict(B=1, H=2, L=512, C=16, Lq=64, U=64, keep_frac=0.3, causal_user=True),
    dict(B=2, H=3, L=1000, C=37, Lq=70, U=70, keep_frac=0.25, causal_user=True),     # ragged everything
    dict(B=1, H=2, L=2048, C=2048, Lq=33, U=10, keep_frac=0.3, causal_user=False),   # many empty clusters: wide spans
    dict(B=1, H=1, L=300, C=8, Lq=5, U=0, keep_frac=0.5, causal_user=False),         # no user keys
    dict(B=1, H=2, L=4096, C=128, Lq=200, U=200, keep_frac=0.125, causal_user=True),
])
def test_prefill_small(sq, oracle, case):
    w = wl.calibrate(wl.make_workload("prefill_small", seed=21, threads=2, **case), oracle.scores)
    P = sq.upload(w)
    run_prefill(sq, w, P)
    compare_prefill(oracle, w, P, f"prefill{case}")


def test_prefill_empty_and_keep_all(sq, oracle):
    w = wl.make_workload("prefill_edge", B=1, H=2, L=700, C=20, Lq=40, U=40, keep_frac=0.5, causal_user=True, seed=22,
                         threads=1)
    w.thresh = np.full(w.H, 2.0, np.float32)              # nothing kept: causal attention over the user keys only
    P = sq.upload(w); run_prefill(sq, w, P)
    assert (P.n_keys.cpu().numpy() == 0).all()
    compare_prefill(oracle, w, P, "prefill-empty")
    w.thresh = np.full(w.H, -1.0, np.float32)             # everything kept: dense attention
    P = sq.upload(w); run_prefill(sq, w, P)
    assert (P.n_keys.cpu().numpy() == w.L).all()
    compare_prefill(oracle, w, P, "prefill-keep-all")
    from oracle import literal
    for h in range(w.H):
        t = 17
        K = np.concatenate([w.K_fixed[h], w.K_user[0, h, :t + 1]]); V = np.concatenate([w.V_fixed[h], w.V_user[0, h, :t + 1]])
        ref, _ = literal.dense_attention(w.q[0, h, t:t + 1], K, V, w.sm_scale)
        assert np.abs(P.out[0, h, t].cpu().numpy().astype(np.float64) - ref[0]).max() <= ATTN_ATOL


def banded_keep(w, rng, band, extra, qb=64):
    """Keep sets that follow the query's position: the 64 queries of a query block share a band of clusters (plus
    `extra` stray clusters per block, and a few queries that keep nothing), so most key blocks are kept by no
    query of the block."""
    gk = np.zeros((w.B, w.H, w.Lq, w.C), bool)
    for b in range(w.B):
        for h in range(w.H):
            for g in range(0, w.Lq, qb):
                lo = int(rng.integers(0, max(1, w.C - band)))
                stray = rng.integers(0, w.C, size=extra)
                for t in range(g, min(g + qb, w.Lq)):
                    if rng.random() < 0.05:
                        continue
                    a = lo + int(rng.integers(0, band // 2)); e = a + int(rng.integers(1, band // 2 + 1))
                    gk[b, h, t, a:e] = True
                    if extra:
                        gk[b, h, t, stray[rng.integers(0, extra)]] = True
    return gk


@pytest.mark.parametrize("case", [
    dict(B=1, H=2, L=8192, C=512, Lq=200, U=64, band=48, extra=2, causal_user=True),
    dict(B=2, H=2, L=5000, C=300, Lq=130, U=0, band=30, extra=0, causal_user=False),      # ragged, no user keys
    dict(B=1, H=2, L=5000, C=300, Lq=200, U=0, band=30, extra=0, causal_user=False, blank=(64, 128)),   # a query block with nothing to attend to
    dict(B=1, H=1, L=4096, C=4096, Lq=64, U=40, band=400, extra=3, causal_user=True),     # empty clusters: wide blocks
    dict(B=1, H=2, L=40000, C=2000, Lq=100, U=30, band=150, extra=4, causal_user=True),   # 625 key blocks: the list is built in rounds
])
def test_prefill_masks_that_follow_position(sq, oracle, case):
    """Explicit keep masks under which most (query block, key block) pairs hold no kept key: the kernel that walks only
    the listed blocks does the work (its rule: an eighth of the pairs or more can be skipped)."""
    case = dict(case); band = case.pop("band"); extra = case.pop("extra"); blank = case.pop("blank", None)
    w = wl.make_workload("prefill_banded", seed=23, threads=2, keep_frac=0.1, **case)
    rng = np.random.default_rng(5)
    gk = banded_keep(w, rng, band, extra)
    if blank:
        gk[:, :, blank[0]:blank[1]] = False
    # share of (query block, key block) pairs without a kept key
    nblk = (w.L + 63) // 64
    skip = tot = 0
    for h in range(w.H):
        cid = np.repeat(np.arange(w.C), w.sizes[h])
        for b in range(w.B):
            for g in range(0, w.Lq, 64):
                kept_keys = gk[b, h, g:g + 64].any(0)[cid]
                need = np.add.reduceat(kept_keys, np.arange(0, w.L, 64)) > 0
                skip += nblk - int(need.sum()); tot += nblk
    assert skip * 8 >= tot, (skip, tot)
    W = (w.C + 31) // 32
    bits = np.zeros((w.B, w.H, w.Lq, W * 32), bool); bits[..., :w.C] = gk
    words = (bits.reshape(w.B, w.H, w.Lq, W, 32) * (1 << np.arange(32, dtype=np.uint64))).sum(-1).astype(np.uint32)
    P = sq.upload(w)
    P.keep_mask.copy_(torch.from_numpy(words.view(np.int32)))
    ws = sq.workspace(P.shape, sq.SQ_CALL_ATTN_PREFILL, P.q.device)
    sq.sq_sparse_attn_prefill(P.shape, P.q, P.K_fixed, P.V_fixed, P.offsets, P.keep_mask, P.K_user, P.V_user, P.out,
                              P.lse, ws)
    torch.cuda.synchronize()
    R = (w.B, w.H, w.Lq)
    cap = int(gk.sum(-1).max()) + 1
    ranges = np.zeros((*R, cap, 2), np.int32); n_r = np.zeros(R, np.int32)
    for b, h, t in np.ndindex(*R):
        ranges[b, h, t], n_r[b, h, t] = ranges_from_keep(gk[b, h, t], w.offsets[h], w.sizes[h], cap)
    out, lse = oracle.sparse_attn(w.q, w.K_fixed, w.V_fixed, ranges, n_r, w.K_user, w.V_user, w.sm_scale,
                                  causal_user=w.causal_user)
    err = np.abs(P.out.cpu().numpy().astype(np.float64) - out).max()
    assert err <= ATTN_ATOL, f"{case}: attention max-abs error {err}"
    np.testing.assert_allclose(P.lse.cpu().numpy(), lse, atol=2e-4, rtol=1e-5)
    print(f"banded {case}: skippable pairs {skip}/{tot}, max-abs err {err:.2e}", flush=True)


def test_cfg4_sparse_prefill_32k(sq, oracle):
    print("cfg4: generating", flush=True)
    w = wl.calibrate(wl.make_config("cfg4_prefill_32k", threads=16), oracle.scores)
    P = sq.upload(w)
    print("cfg4: running", flush=True)
    run_prefill(sq, w, P)
    print("cfg4: comparing (selection and attention on all 32768 rows)", flush=True)
    err = compare_prefill(oracle, w, P, "cfg4")
    print("cfg4 attention max-abs err", err, "mean keep", P.n_keys.float().mean().item() / w.L, flush=True)


# ---- selection on averaged scores + attention over one shared kept set (Appendix D, "Prefill Stage") ----------

def mean_thresholds(oracle, w):
    """Per-head thresholds on the AVERAGED scores that keep about w.keep_frac of the keys (oracle scores)."""
    x, m, D = oracle.centroid_score(w.q, w.centroids, w.sizes, w.sm_scale)
    sbar = oracle.select_mean(x, m, D, np.zeros(w.H, np.float32), w.sizes, w.offsets, want_scores=True)[4]
    thr = np.empty(w.H, np.float32)
    for h in range(w.H):
        live = np.tile(w.sizes[h] > 0, w.B)
        thr[h] = wl._cut(sbar[:, h].ravel()[live], np.tile(w.sizes[h], w.B)[live], w.keep_frac * w.L * w.B)
    return thr, (x, m, D)


def run_prefill_mean(sq, w, P):
    sh = P.shape
    d = P.q.device
    W = (w.C + 31) // 32
    mask = torch.zeros(w.B, w.H, W, dtype=torch.int32, device=d)
    ranges = torch.zeros(w.B, w.H, w.C, 2, dtype=torch.int32, device=d)
    nr = torch.zeros(w.B, w.H, dtype=torch.int32, device=d)
    nk = torch.zeros(w.B, w.H, dtype=torch.int32, device=d)
    sq.sq_centroid_score(sh, P.q, P.centroids, P.sizes, P.logits, P.row_max, P.denom)
    sq.sq_select_mean(sh, P.logits, P.row_max, P.denom, P.thresh, P.sizes, P.offsets, mask, ranges, nr, nk,
                      sq.workspace(sh, sq.SQ_CALL_SELECT_MEAN, d))
    sq.sq_sparse_attn_prefill_shared(sh, P.q, P.K_fixed, P.V_fixed, ranges, nr, nk, P.K_user, P.V_user, P.out, P.lse,
                                     sq.workspace(sh, sq.SQ_CALL_ATTN_PREFILL_SHARED, d))
    torch.cuda.synchronize()
    return mask.cpu().numpy(), ranges.cpu().numpy(), nr.cpu().numpy(), nk.cpu().numpy()


def compare_prefill_mean(oracle, w, P, got, stats, label, sample=None, rng=None):
    from oracle import literal
    mask, ranges, nr, nk = got
    x, m, D = stats
    omask = oracle.select_mean(x, m, D, w.thresh, w.sizes, w.offsets)[0]
    gk, ok = unpack_mask(mask, w.C), unpack_mask(omask, w.C)
    listed = []
    for b, h, c in np.argwhere(gk != ok):                  # disagreements must sit next to the threshold
        sbar = literal.select_mean(w.q[b, h], w.centroids[h], w.sizes[h], w.thresh[h], w.sm_scale)[1]
        assert literal.near_threshold(sbar[c], w.thresh[h]), (
            f"{label} cluster {(b, h, c)}: gpu={gk[b, h, c]} oracle={ok[b, h, c]} mean score {sbar[c]:.9e} "
            f"T={w.thresh[h]:.9e}")
        listed.append((int(b), int(h), int(c), float(sbar[c]), float(w.thresh[h])))
    if listed:
        print(f"[near-threshold clusters {label}]", listed)
    np.testing.assert_array_equal(nk, (gk * w.sizes[None]).sum(-1))
    if ranges is None:                                    # (the whole-step call returns mask and counts only)
        nr = gk.sum(-1).astype(np.int32)
        ranges = np.zeros((w.B, w.H, w.C, 2), np.int32)
        for b in range(w.B):
            for h in range(w.H):
                ranges[b, h], _ = ranges_from_keep(gk[b, h], w.offsets[h], w.sizes[h], w.C)
    np.testing.assert_array_equal(nr, gk.sum(-1))
    for b in range(w.B):
        for h in range(w.H):
            ids = np.flatnonzero(gk[b, h])
            np.testing.assert_array_equal(ranges[b, h, :len(ids)], np.stack([w.offsets[h, ids], w.sizes[h, ids]], 1)
                                          if len(ids) else np.zeros((0, 2), np.int32))
    # attention over the GPU's own (validated) set, the same ranges for every query token of a (b, h)
    R = (w.B, w.H, w.Lq)
    sel = np.ones(R, bool)
    if sample is not None:
        sel = np.zeros(R, bool)
        sel.ravel()[rng.choice(sel.size, size=sample, replace=False)] = True
        sel[:, :, 0] = True; sel[:, :, -1] = True
    cap = max(1, int(nr.max()))
    rr = np.ascontiguousarray(np.broadcast_to(ranges[:, :, None, :cap], (*R, cap, 2)))
    nn = np.ascontiguousarray(np.broadcast_to(nr[:, :, None], R))
    out, lse = oracle.sparse_attn(w.q, w.K_fixed, w.V_fixed, rr, nn, w.K_user, w.V_user, w.sm_scale,
                                  causal_user=w.causal_user, row_sel=sel)
    err = np.abs(P.out.cpu().numpy().astype(np.float64)[sel] - out[sel]).max()
    assert err <= ATTN_ATOL, f"{label}: attention max-abs error {err} over {sel.sum()} rows"
    glse = P.lse.cpu().numpy()[sel]
    fin = np.isfinite(lse[sel])
    assert (np.isneginf(glse) == ~fin).all()
    np.testing.assert_allclose(glse[fin], lse[sel][fin], atol=2e-4, rtol=1e-5)
    return err


@pytest.mark.parametrize("case", [
    dict(B=1, H=2, L=512, C=16, Lq=64, U=64, keep_frac=0.3, causal_user=True),
    dict(B=2, H=3, L=1000, C=37, Lq=70, U=70, keep_frac=0.25, causal_user=True),     # ragged everything
    dict(B=1, H=2, L=2048, C=2048, Lq=33, U=10, keep_frac=0.3, causal_user=False),   # more clusters than one step
    dict(B=1, H=1, L=300, C=8, Lq=5, U=0, keep_frac=0.5, causal_user=False),         # no user keys
    dict(B=1, H=2, L=4096, C=128, Lq=200, U=200, keep_frac=0.125, causal_user=True),
    dict(B=1, H=1, L=5000, C=50, Lq=130, U=3, keep_frac=0.6, causal_user=True),      # long kept list with a ragged tail
])
def test_prefill_mean_selection_small(sq, oracle, case):
    w = wl.make_workload("prefill_mean", seed=23, threads=2, **case)
    w.thresh, stats = mean_thresholds(oracle, w)
    P = sq.upload(w)
    got = run_prefill_mean(sq, w, P)
    compare_prefill_mean(oracle, w, P, got, stats, f"prefill-mean{case}")


def test_prefill_mean_selection_extremes(sq, oracle):
    base = dict(B=1, H=2, L=700, C=20, Lq=40, U=40, keep_frac=0.5, causal_user=True, seed=24, threads=1)
    for T, label in [(2.0, "nothing kept"), (-1.0, "everything kept")]:
        w = wl.make_workload("prefill_mean_edge", **base)
        w.thresh = np.full(w.H, T, np.float32)
        stats = oracle.centroid_score(w.q, w.centroids, w.sizes, w.sm_scale)
        P = sq.upload(w)
        got = run_prefill_mean(sq, w, P)
        assert (got[3] == (0 if T > 0 else w.L)).all()
        compare_prefill_mean(oracle, w, P, got, stats, f"prefill-mean {label}")
    # nothing kept and no user keys: zero output, lse = -inf
    w = wl.make_workload("prefill_mean_void", **dict(base, U=0))
    w.thresh = np.full(w.H, 2.0, np.float32)
    P = sq.upload(w)
    P.out.fill_(7.0)
    run_prefill_mean(sq, w, P)
    assert (P.out.cpu().numpy() == 0).all() and np.isneginf(P.lse.cpu().numpy()).all()


def test_cfg4_shape_prefill_mean_selection(sq, oracle):
    print("cfg4 (averaged selection): generating", flush=True)
    w = wl.make_config("cfg4_prefill_32k", threads=16)
    w.thresh, stats = mean_thresholds(oracle, w)
    P = sq.upload(w)
    print("cfg4 (averaged selection): running", flush=True)
    got = run_prefill_mean(sq, w, P)
    print("cfg4 (averaged selection): comparing all 32768 rows", flush=True)
    err = compare_prefill_mean(oracle, w, P, got, stats, "cfg4-mean")
    print("cfg4-mean attention max-abs err", err, "keep", got[3].mean() / w.L, flush=True)


# ---- whole prefill steps (two-pass lookup with nothing materialised + attention) ---------------------------------

STEP_CASES = [
    dict(B=1, H=2, L=512, C=16, Lq=64, U=64, keep_frac=0.3, causal_user=True),
    dict(B=2, H=3, L=1000, C=37, Lq=70, U=70, keep_frac=0.25, causal_user=True),     # ragged: C % 16, Lq % 16, words
    dict(B=1, H=2, L=2048, C=2048, Lq=33, U=10, keep_frac=0.3, causal_user=False),   # many empty clusters
    dict(B=1, H=1, L=300, C=8, Lq=5, U=0, keep_frac=0.5, causal_user=False),         # fewer clusters than a tile
    dict(B=1, H=2, L=4096, C=128, Lq=200, U=200, keep_frac=0.125, causal_user=True),
]


def run_prefill_step(sq, w, P):
    sh = P.shape
    sq.sq_prefill_step(sh, P.q, P.centroids, P.sizes, P.offsets, P.thresh, P.K_fixed, P.V_fixed, P.K_user, P.V_user,
                       P.out, P.lse, P.keep_mask, P.n_keys, sq.workspace(sh, sq.SQ_CALL_PREFILL_STEP, P.q.device))
    torch.cuda.synchronize()


def run_prefill_mean_step(sq, w, P):
    sh, d = P.shape, P.q.device
    mask = torch.zeros(w.B, w.H, (w.C + 31) // 32, dtype=torch.int32, device=d)
    nk = torch.zeros(w.B, w.H, dtype=torch.int32, device=d)
    sq.sq_prefill_mean_step(sh, P.q, P.centroids, P.sizes, P.offsets, P.thresh, P.K_fixed, P.V_fixed, P.K_user,
                            P.V_user, P.out, P.lse, mask, nk, sq.workspace(sh, sq.SQ_CALL_PREFILL_MEAN_STEP, d))
    torch.cuda.synchronize()
    return mask.cpu().numpy(), None, None, nk.cpu().numpy()


@pytest.mark.parametrize("case", STEP_CASES)
def test_prefill_step_small(sq, oracle, case):
    w = wl.calibrate(wl.make_workload("prefill_step", seed=25, threads=2, **case), oracle.scores)
    P = sq.upload(w)
    run_prefill_step(sq, w, P)
    compare_prefill(oracle, w, P, f"prefill-step{case}", logits=False)


@pytest.mark.parametrize("case", STEP_CASES)
def test_prefill_mean_step_small(sq, oracle, case):
    w = wl.make_workload("prefill_mean_step", seed=26, threads=2, **case)
    w.thresh, stats = mean_thresholds(oracle, w)
    P = sq.upload(w)
    got = run_prefill_mean_step(sq, w, P)
    compare_prefill_mean(oracle, w, P, got, stats, f"prefill-mean-step{case}")


def test_prefill_step_queries_alike_within_a_block(sq, oracle):
    """The whole step on queries that resemble their neighbours (each block of 64 tokens shares a direction, as
    consecutive tokens of a prompt do): the selections of a block overlap, most key blocks are kept by no token of it,
    and the step's attention runs through the kernel that walks only the listed blocks."""
    w = wl.make_workload("prefill_alike", seed=29, threads=2, B=1, H=2, L=8192, C=512, Lq=192, U=64, keep_frac=0.05,
                         causal_user=True)
    rng = np.random.default_rng(9)
    q = w.q.astype(np.float32)
    for h in range(w.H):
        for g in range(0, w.Lq, 64):
            base = q[0, h, g]                                 # the block's first token gives the direction
            n = min(64, w.Lq - g)
            q[0, h, g:g + n] = base[None, :] + 0.05 * np.abs(base).mean() * rng.standard_normal((n, w.d))
    w.q = q.astype(np.float16)
    w = wl.calibrate(w, oracle.scores)
    # the scenario itself, from the oracle's selection: at least an eighth of the (query block, key block) pairs are empty
    x, m, D = oracle.centroid_score(w.q, w.centroids, w.sizes, w.sm_scale)
    mask, _, _, _ = oracle.select(x, m, D, w.thresh, w.sizes, w.offsets)
    keep = unpack_mask(mask, w.C)
    nblk = (w.L + 63) // 64
    skip = tot = 0
    for h in range(w.H):
        cid = np.repeat(np.arange(w.C), w.sizes[h])
        for g in range(0, w.Lq, 64):
            need = np.add.reduceat(keep[0, h, g:g + 64].any(0)[cid], np.arange(0, w.L, 64)) > 0
            skip += nblk - int(need.sum()); tot += nblk
    assert skip * 8 >= tot, (skip, tot)
    P = sq.upload(w)
    run_prefill_step(sq, w, P)
    err = compare_prefill(oracle, w, P, "prefill-step-alike", logits=False)
    print(f"queries alike within a block: skippable pairs {skip}/{tot}, max-abs err {err:.2e}", flush=True)


def test_prefill_steps_extremes_and_optional_outputs(sq, oracle):
    base = dict(B=1, H=2, L=700, C=20, Lq=40, U=40, keep_frac=0.5, causal_user=True, seed=27, threads=1)
    for T in (2.0, -1.0):                                  # nothing kept / everything kept
        w = wl.make_workload("prefill_step_edge", **base)
        w.thresh = np.full(w.H, T, np.float32)
        P = sq.upload(w)
        run_prefill_step(sq, w, P)
        assert (P.n_keys.cpu().numpy() == (0 if T > 0 else w.L)).all()
        compare_prefill(oracle, w, P, f"prefill-step T={T}", logits=False)
        ref = P.out.clone()
        stats = oracle.centroid_score(w.q, w.centroids, w.sizes, w.sm_scale)
        got = run_prefill_mean_step(sq, w, P)
        assert (got[3] == (0 if T > 0 else w.L)).all()
        compare_prefill_mean(oracle, w, P, got, stats, f"prefill-mean-step T={T}")
        # with one kept set for all tokens (all or nothing) the two rules select the same keys
        assert (P.out.float() - ref.float()).abs().max().item() <= 1e-3
    # optional outputs left out
    w = wl.calibrate(wl.make_workload("prefill_step_opt", **base), oracle.scores)
    P = sq.upload(w)
    run_prefill_step(sq, w, P)
    ref = P.out.clone()
    P.out.zero_()
    sq.sq_prefill_step(P.shape, P.q, P.centroids, P.sizes, P.offsets, P.thresh, P.K_fixed, P.V_fixed, P.K_user,
                       P.V_user, P.out, None, None, None, sq.workspace(P.shape, sq.SQ_CALL_PREFILL_STEP, P.q.device))
    torch.cuda.synchronize()
    assert torch.equal(P.out, ref)


def test_cfg4_prefill_steps(sq, oracle):
    print("cfg4 (whole steps): generating", flush=True)
    w = wl.calibrate(wl.make_config("cfg4_prefill_32k", threads=16), oracle.scores)
    P = sq.upload(w)
    run_prefill_step(sq, w, P)
    print("cfg4 (whole steps): comparing all 32768 rows", flush=True)
    err = compare_prefill(oracle, w, P, "cfg4-step", logits=False)
    print("cfg4 sq_prefill_step attention max-abs err", err, flush=True)
    w.thresh, stats = mean_thresholds(oracle, w)
    P = sq.upload(w)
    got = run_prefill_mean_step(sq, w, P)
    print("cfg4 (whole steps, averaged selection): comparing all 32768 rows", flush=True)
    err = compare_prefill_mean(oracle, w, P, got, stats, "cfg4-mean-step")
    print("cfg4 sq_prefill_mean_step attention max-abs err", err, "keep", got[3].mean() / w.L, flush=True)
