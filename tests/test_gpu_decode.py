"""GPU parity: the decode path through the C ABI against the CPU oracle (configs 1-3 and edge cases)."""
import numpy as np
import pytest
import torch

from gpu_util import (ATTN_ATOL, DENOM_RTOL, LOGIT_ATOL, check_selection, dev, expand_ranges, oracle_one_level,
                      ranges_from_keep, unpack_mask)
from paper_2411_09688_amd import workload as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sq():
    from paper_2411_09688_amd import binding
    binding.lib()
    return binding


def run_separate(sq, w, P):
    """sq_centroid_score -> sq_select -> sq_sparse_attn_decode, each through the C ABI."""
    sh = P.shape
    sq.sq_centroid_score(sh, P.q, P.centroids, P.sizes, P.logits, P.row_max, P.denom)
    sq.sq_select(sh, P.logits, P.row_max, P.denom, P.thresh, P.sizes, P.offsets, P.keep_mask, P.ranges, P.n_ranges,
                 P.n_keys)
    ws = sq.workspace(sh, sq.SQ_CALL_ATTN_DECODE, P.q.device)
    sq.sq_sparse_attn_decode(sh, P.q, P.K_fixed, P.V_fixed, P.ranges, P.n_ranges, P.n_keys, P.K_user, P.V_user, P.out,
                             P.lse, ws)
    torch.cuda.synchronize()


def compare_decode(oracle, w, P, ref, label):
    C = w.C
    np.testing.assert_allclose(P.logits.cpu().numpy(), ref["logits"], atol=LOGIT_ATOL, rtol=0)
    np.testing.assert_allclose(P.row_max.cpu().numpy(), ref["row_max"], atol=LOGIT_ATOL, rtol=0)
    np.testing.assert_allclose(P.denom.cpu().numpy(), ref["denom"], rtol=DENOM_RTOL)
    gk = unpack_mask(P.keep_mask.cpu().numpy(), C)
    ok = unpack_mask(ref["mask"], C)
    listed = check_selection(w, gk, ok, w.thresh, label=label)
    nr, nk = P.n_ranges.cpu().numpy(), P.n_keys.cpu().numpy()
    np.testing.assert_array_equal(nr, gk.sum(-1))
    np.testing.assert_array_equal(nk, (gk * w.sizes[None, :, None, :]).sum(-1))
    rg = P.ranges.cpu().numpy()
    for b in range(w.B):
        for h in range(w.H):
            ids = np.flatnonzero(gk[b, h, 0])
            exp = np.stack([w.offsets[h, ids], w.sizes[h, ids]], 1) if len(ids) else np.zeros((0, 2), np.int32)
            np.testing.assert_array_equal(rg[b, h, 0, :len(ids)], exp)
    # Attention is compared on the GPU's own (validated) selection: identical to the oracle's unless a
    # near-threshold cluster was listed above.
    if listed:
        ranges = np.zeros_like(ref["ranges"]); n_r = np.zeros_like(ref["n_ranges"])
        for b in range(w.B):
            for h in range(w.H):
                ranges[b, h, 0], n_r[b, h, 0] = ranges_from_keep(gk[b, h, 0], w.offsets[h], w.sizes[h], C)
    else:
        ranges, n_r = ref["ranges"], ref["n_ranges"]
    out, lse = oracle.sparse_attn(w.q, w.K_fixed, w.V_fixed, ranges, n_r, w.K_user, w.V_user, w.sm_scale)
    err = np.abs(P.out.cpu().numpy().astype(np.float64) - out).max()
    assert err <= ATTN_ATOL, f"{label}: attention max-abs error {err}"
    np.testing.assert_allclose(P.lse.cpu().numpy(), lse, atol=1e-4, rtol=1e-5)
    return out, lse


def fused_matches(sq, w, P):
    """sq_decode_step against the three separate calls.  The step scores the centroids with its own kernel (another
    fp32 summation order than sq_centroid_score), so a cluster whose score sits within rounding of the threshold may be
    decided differently: every difference must lie in the near-threshold band.  Rows with identical selections have
    attention outputs equal up to the rounding of a different split of the keys over workgroups."""
    sh = P.shape
    out2 = torch.zeros_like(P.out); lse2 = torch.zeros_like(P.lse)
    mask2 = torch.zeros_like(P.keep_mask); nk2 = torch.zeros_like(P.n_keys)
    ws = sq.workspace(sh, sq.SQ_CALL_DECODE_STEP, P.q.device)
    sq.sq_decode_step(sh, P.q, P.centroids, P.sizes, P.offsets, P.thresh, P.K_fixed, P.V_fixed, P.K_user, P.V_user,
                      out2, lse2, mask2, nk2, ws)
    torch.cuda.synchronize()
    g2, g1 = unpack_mask(mask2.cpu().numpy(), w.C), unpack_mask(P.keep_mask.cpu().numpy(), w.C)
    check_selection(w, g2, g1, w.thresh, label="step vs separate calls")
    np.testing.assert_array_equal(nk2.cpu().numpy(), (g2 * w.sizes[None, :, None, :]).sum(-1))
    same = torch.from_numpy((g2 == g1).all(-1)).to(P.out.device)          # [B,H,1]
    if same.any():
        assert (out2.float() - P.out.float()).abs().amax(-1)[same].max().item() <= 1e-3
        torch.testing.assert_close(lse2[same], P.lse[same], atol=1e-5, rtol=1e-6)


@pytest.fixture(scope="module")
def cfg1(oracle):
    return wl.calibrate(wl.make_config("cfg1_tiny_decode"), oracle.scores)


def test_cfg1_tiny_decode(sq, oracle, cfg1):
    w = cfg1
    P = sq.upload(w)
    run_separate(sq, w, P)
    compare_decode(oracle, w, P, oracle_one_level(oracle, w), "cfg1")
    fused_matches(sq, w, P)


def test_cfg2_llama7b_decode_32k(sq, oracle):
    print("cfg2: generating", flush=True)
    w = wl.calibrate(wl.make_config("cfg2_decode_32k"), oracle.scores)
    P = sq.upload(w)
    print("cfg2: running", flush=True)
    run_separate(sq, w, P)
    compare_decode(oracle, w, P, oracle_one_level(oracle, w), "cfg2")
    fused_matches(sq, w, P)
    print("cfg2 keep fraction per head:", np.round(P.n_keys.cpu().numpy().ravel() / w.L, 3), flush=True)
    # the entry point the benchmark times, at the benchmarked size, against the oracle directly
    step_against_oracle(sq, oracle, w, "cfg2 sq_decode_step")


def test_cfg2_shape_single_global_threshold(sq, oracle):
    """Config 2's shape with heads of different score skewness under ONE threshold for all heads (Section 3.2,
    appendix "Attention Score Skewness"): the heads keep very different numbers of keys, which is the case the equal
    split of the kept keys over the compute units (Section 4.2) exists for.  Whole step against the oracle."""
    w = wl.calibrate(wl.make_config("cfg2_decode_32k", head_skew=0.4), oracle.scores, global_threshold=True)
    assert np.ptp(w.thresh) == 0
    step_against_oracle(sq, oracle, w, "cfg2 shape, one global threshold")
    P = sq.upload(w)
    ws = sq.workspace(P.shape, sq.SQ_CALL_DECODE_STEP, P.q.device)
    sq.sq_decode_step(P.shape, P.q, P.centroids, P.sizes, P.offsets, P.thresh, P.K_fixed, P.V_fixed, P.K_user,
                      P.V_user, P.out, P.lse, P.keep_mask, P.n_keys, ws)
    torch.cuda.synchronize()
    frac = P.n_keys.cpu().numpy().ravel() / w.L
    print("global threshold: keep fraction per head", np.round(frac, 3), "overall", round(float(frac.mean()), 4), flush=True)
    assert frac.max() > 5 * max(frac.min(), 1e-4)          # the heads do differ


def test_cfg3_batched_decode_shared_context(sq, oracle):
    print("cfg3: generating", flush=True)
    w = wl.calibrate(wl.make_config("cfg3_batched_decode_32k"), oracle.scores)
    P = sq.upload(w)
    print("cfg3: running", flush=True)
    run_separate(sq, w, P)
    compare_decode(oracle, w, P, oracle_one_level(oracle, w), "cfg3")
    fused_matches(sq, w, P)
    step_against_oracle(sq, oracle, w, "cfg3 sq_decode_step")


def test_keep_all_equals_dense_attention(sq, oracle, cfg1):
    # A negative threshold keeps every non-empty cluster: the path must reproduce dense attention.
    w = cfg1
    P = sq.upload(w, thresh=np.full(w.H, -1.0, np.float32))
    run_separate(sq, w, P)
    assert (P.n_keys.cpu().numpy() == w.L).all()
    from oracle import literal
    for h in range(w.H):
        K = np.concatenate([w.K_fixed[h], w.K_user[0, h]]); V = np.concatenate([w.V_fixed[h], w.V_user[0, h]])
        ref, lse = literal.dense_attention(w.q[0, h], K, V, w.sm_scale)
        assert np.abs(P.out[0, h].cpu().numpy().astype(np.float64) - ref).max() <= ATTN_ATOL
        np.testing.assert_allclose(P.lse[0, h].cpu().numpy(), lse, atol=1e-4)


@pytest.mark.parametrize("case", [
    dict(B=1, H=1, L=5, C=1, U=0, keep_frac=1.0),                # single cluster, no user keys
    dict(B=2, H=3, L=777, C=37, U=1, keep_frac=0.3),             # ragged: C not a multiple of 32, odd L, U=1
    dict(B=3, H=2, L=3000, C=100, U=300, keep_frac=0.5),         # several chunks with a ragged tail, 2 user chunks
    dict(B=1, H=2, L=2048, C=2048, U=17, keep_frac=0.2),         # one key per cluster on average (many empty clusters)
    dict(B=17, H=1, L=1500, C=65, U=40, keep_frac=0.25),         # more than 16 sequences: two query tiles
])
def test_ragged_shapes(sq, oracle, case):
    w = wl.calibrate(wl.make_workload("ragged", Lq=1, seed=3, threads=2, **case), oracle.scores)
    P = sq.upload(w)
    run_separate(sq, w, P)
    compare_decode(oracle, w, P, oracle_one_level(oracle, w), f"ragged{case}")
    fused_matches(sq, w, P)


def test_empty_selection_and_no_user_keys(sq, oracle):
    w = wl.make_workload("empty", B=2, H=2, L=512, C=16, Lq=1, U=0, keep_frac=0.5, seed=4, threads=1)
    w.thresh = np.full(w.H, 2.0, np.float32)           # above every score: nothing is kept
    P = sq.upload(w)
    P.out.fill_(7.0)
    run_separate(sq, w, P)
    assert (P.n_keys.cpu().numpy() == 0).all() and (P.n_ranges.cpu().numpy() == 0).all()
    assert (P.keep_mask.cpu().numpy() == 0).all()
    assert (P.out.cpu().numpy() == 0).all() and np.isneginf(P.lse.cpu().numpy()).all()
    fused_matches(sq, w, P)
    # nothing kept but user keys present: attention over the user keys only
    w2 = wl.make_workload("empty_u", B=1, H=2, L=512, C=16, Lq=1, U=9, keep_frac=0.5, seed=5, threads=1)
    w2.thresh = np.full(w2.H, 2.0, np.float32)
    P2 = sq.upload(w2)
    run_separate(sq, w2, P2)
    compare_decode(oracle, w2, P2, oracle_one_level(oracle, w2), "user-only")


def step_against_oracle(sq, oracle, w, label, keep_mask=True):
    """sq_decode_step alone, compared with the oracle directly (selection, counts, attention)."""
    P = sq.upload(w)
    sh = P.shape
    ws = sq.workspace(sh, sq.SQ_CALL_DECODE_STEP, P.q.device)
    P.out.fill_(7.0)
    sq.sq_decode_step(sh, P.q, P.centroids, P.sizes, P.offsets, P.thresh, P.K_fixed, P.V_fixed, P.K_user, P.V_user,
                      P.out, P.lse, P.keep_mask if keep_mask else None, P.n_keys, ws)
    torch.cuda.synchronize()
    ref = oracle_one_level(oracle, w)
    ok = unpack_mask(ref["mask"], w.C)
    if keep_mask:
        gk = unpack_mask(P.keep_mask.cpu().numpy(), w.C)
        listed = check_selection(w, gk, ok, w.thresh, label=label)
    else:
        gk, listed = ok, []
    np.testing.assert_array_equal(P.n_keys.cpu().numpy(), (gk * w.sizes[None, :, None, :]).sum(-1))
    ranges = np.zeros_like(ref["ranges"]); n_r = np.zeros_like(ref["n_ranges"])
    for b in range(w.B):
        for h in range(w.H):
            ranges[b, h, 0], n_r[b, h, 0] = ranges_from_keep(gk[b, h, 0], w.offsets[h], w.sizes[h], w.C)
    out, lse = oracle.sparse_attn(w.q, w.K_fixed, w.V_fixed, ranges, n_r, w.K_user, w.V_user, w.sm_scale)
    err = np.abs(P.out.cpu().numpy().astype(np.float64) - out).max()
    assert err <= ATTN_ATOL, f"{label}: attention max-abs error {err}"
    got = P.lse.cpu().numpy()
    fin = np.isfinite(lse)
    assert (np.isneginf(got) == ~fin).all()
    np.testing.assert_allclose(got[fin], lse[fin], atol=1e-4, rtol=1e-5)
    return listed


@pytest.mark.parametrize("case", [
    dict(B=8, H=2, L=900, C=30, U=5, keep_frac=0.3),               # smallest batch that takes the shared-context kernels
    dict(B=11, H=3, L=3000, C=100, U=300, keep_frac=0.5),          # partial group; user chunks with a ragged tail
    dict(B=16, H=2, L=2000, C=50, U=0, keep_frac=0.2),             # one full group, no user keys
    dict(B=33, H=1, L=1500, C=65, U=40, keep_frac=0.25),           # three groups, the last with one sequence
    dict(B=9, H=2, L=4096, C=2048, U=17, keep_frac=0.2),           # more clusters than one selection step holds
    dict(B=8, H=1, L=70000, C=300, U=130, keep_frac=0.6),          # several workgroups per union row, long clusters
    dict(B=2, H=2, L=900, C=30, U=5, keep_frac=0.3),               # below the shared-context threshold: per-row kernels
    dict(B=7, H=2, L=2500, C=80, U=140, keep_frac=0.4),            # the largest batch on the per-row kernels
])
def test_shared_context_step_against_oracle(sq, oracle, case):
    w = wl.calibrate(wl.make_workload("shared", Lq=1, seed=11, threads=4, **case), oracle.scores)
    step_against_oracle(sq, oracle, w, f"shared{case}")


@pytest.mark.parametrize("case", [
    dict(B=1, H=2, L=6000, C=4096, U=70, keep_frac=0.3),          # most clusters the key-index step takes
    dict(B=1, H=2, L=6000, C=4100, U=70, keep_frac=0.3),          # one step past it: the work-list kernels
    dict(B=4, H=256, L=300, C=20, U=3, keep_frac=0.4),            # 1024 query rows: the most the key-index step takes
    dict(B=4, H=257, L=300, C=20, U=3, keep_frac=0.4),            # 1028 rows: the work-list kernels
    dict(B=3, H=5, L=700, C=40, U=64, keep_frac=0.02),            # rows that keep (almost) nothing; one whole user piece
    dict(B=2, H=3, L=900, C=9, U=191, keep_frac=0.95),            # rows that keep (almost) everything; ragged user pieces
])
def test_step_at_key_index_limits(sq, oracle, case):
    w = wl.calibrate(wl.make_workload("limits", Lq=1, seed=21, threads=4, **case), oracle.scores)
    step_against_oracle(sq, oracle, w, f"limits{case}")


def test_shared_context_step_extremes(sq, oracle):
    base = dict(B=10, H=2, L=1024, C=32, Lq=1, U=33, keep_frac=0.5, seed=12, threads=2)
    # every sequence keeps everything: each key is owned by all sequences of the group
    w = wl.make_workload("shared_all", **base)
    w.thresh = np.full(w.H, -1.0, np.float32)
    step_against_oracle(sq, oracle, w, "shared keep-all")
    # nothing kept: user keys only; and without the optional mask output
    w = wl.make_workload("shared_none", **base)
    w.thresh = np.full(w.H, 2.0, np.float32)
    step_against_oracle(sq, oracle, w, "shared keep-none", keep_mask=False)
    # nothing at all to attend to
    w = wl.make_workload("shared_empty", **dict(base, U=0))
    w.thresh = np.full(w.H, 2.0, np.float32)
    P = sq.upload(w)
    P.out.fill_(7.0)
    ws = sq.workspace(P.shape, sq.SQ_CALL_DECODE_STEP, P.q.device)
    sq.sq_decode_step(P.shape, P.q, P.centroids, P.sizes, P.offsets, P.thresh, P.K_fixed, P.V_fixed, P.K_user,
                      P.V_user, P.out, P.lse, P.keep_mask, P.n_keys, ws)
    torch.cuda.synchronize()
    assert (P.out.cpu().numpy() == 0).all() and np.isneginf(P.lse.cpu().numpy()).all()
    assert (P.n_keys.cpu().numpy() == 0).all() and (P.keep_mask.cpu().numpy() == 0).all()


def test_caller_ranges_with_gaps_and_empty_entries(sq, oracle, cfg1):
    # sq_sparse_attn_decode on ranges that did not come from sq_select: merged, with zero-length entries.
    w = cfg1
    P = sq.upload(w)
    rg = np.zeros((w.B, w.H, 1, w.C, 2), np.int32); nr = np.zeros((w.B, w.H, 1), np.int32)
    lists = [[(0, 700), (900, 0), (1000, 1), (1001, 0), (1500, 300)], [(4095, 1)], [], [(10, 0), (20, 0)]]
    for h, lst in enumerate(lists):
        for i, r in enumerate(lst):
            rg[0, h, 0, i] = r
        nr[0, h, 0] = len(lst)
    nk = rg[..., 1].sum(-1).astype(np.int32)
    sh = P.shape
    ws = sq.workspace(sh, sq.SQ_CALL_ATTN_DECODE, P.q.device)
    sq.sq_sparse_attn_decode(sh, P.q, P.K_fixed, P.V_fixed, dev(rg), dev(nr), dev(nk), P.K_user, P.V_user, P.out,
                             P.lse, ws)
    torch.cuda.synchronize()
    out, lse = oracle.sparse_attn(w.q, w.K_fixed, w.V_fixed, rg, nr, w.K_user, w.V_user, w.sm_scale)
    assert np.abs(P.out.cpu().numpy().astype(np.float64) - out).max() <= ATTN_ATOL
    np.testing.assert_allclose(P.lse.cpu().numpy(), lse, atol=1e-4, rtol=1e-5)


def test_errors_are_reported_not_faulted(sq, cfg1):
    P = sq.upload(cfg1)
    sh = P.shape
    with pytest.raises(sq.SqError) as e:
        sq.sq_sparse_attn_decode(sh, P.q, P.K_fixed, P.V_fixed, P.ranges, P.n_ranges, P.n_keys, P.K_user, P.V_user,
                                 P.out, P.lse, torch.empty(256, dtype=torch.uint8, device="cuda:0"))
    assert e.value.code == sq.SQ_ERR_WORKSPACE
    with pytest.raises(sq.SqError) as e:
        sq.sq_centroid_score(sh, None, P.centroids, P.sizes, P.logits, P.row_max, P.denom)
    assert e.value.code == sq.SQ_ERR_INVALID_ARG
