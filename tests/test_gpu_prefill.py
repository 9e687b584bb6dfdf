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


def compare_prefill(oracle, w, P, label, sample=None, rng=None):
    """Selection of every row against the oracle; attention on all rows or on `sample` random rows."""
    C = w.C
    x, m, D = oracle.centroid_score(w.q, w.centroids, w.sizes, w.sm_scale)
    mask, _, nr, nk = oracle.select(x, m, D, w.thresh, w.sizes, w.offsets)
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


def test_cfg4_sparse_prefill_32k(sq, oracle):
    print("cfg4: generating", flush=True)
    w = wl.calibrate(wl.make_config("cfg4_prefill_32k", threads=16), oracle.scores)
    P = sq.upload(w)
    print("cfg4: running", flush=True)
    run_prefill(sq, w, P)
    print("cfg4: comparing (selection on all 32768 rows, attention on 512 sampled rows)", flush=True)
    err = compare_prefill(oracle, w, P, "cfg4", sample=512, rng=np.random.default_rng(4))
    print("cfg4 attention max-abs err", err, "mean keep", P.n_keys.float().mean().item() / w.L, flush=True)
