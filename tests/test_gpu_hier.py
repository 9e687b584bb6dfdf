"""GPU parity: the two-level lookup (sq_hier_select, sq_hier_decode_step) against the CPU oracle."""
import numpy as np
import pytest
import torch

from gpu_util import ATTN_ATOL, dev, ranges_from_keep, unpack_mask
from oracle import literal
from paper_2411_09688_amd import workload as wl
from test_oracle_hier import hier_problem

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sq():
    from paper_2411_09688_amd import binding
    binding.lib()
    return binding


def run_hier_select(sq, B, H, C1, C2, L, q, c1, N1, co, T1, c2, N2, off2, T2, sm_scale, U=0):
    sh = sq.make_shape(B, H, L, C2, 1, U, sm_scale)
    d = "cuda:0"
    t = dict(q=dev(q.reshape(B, H, 1, -1)), c1=dev(c1), N1=dev(N1), co=dev(co), T1=dev(T1), c2=dev(c2), N2=dev(N2),
             off2=dev(off2), T2=dev(T2),
             m1=torch.zeros(B, H, (C1 + 31) // 32, dtype=torch.int32, device=d),
             m2=torch.zeros(B, H, (C2 + 31) // 32, dtype=torch.int32, device=d),
             ranges=torch.zeros(B, H, 1, C2, 2, dtype=torch.int32, device=d),
             nr=torch.zeros(B, H, 1, dtype=torch.int32, device=d), nk=torch.zeros(B, H, 1, dtype=torch.int32, device=d))
    ws = sq.workspace(sh, sq.SQ_CALL_HIER_SELECT, torch.device(d))
    sq.sq_hier_select(sh, C1, t["q"], t["c1"], t["N1"], t["co"], t["T1"], t["c2"], t["N2"], t["off2"], t["T2"],
                      t["m1"], t["m2"], t["ranges"], t["nr"], t["nk"], ws)
    torch.cuda.synchronize()
    return sh, t


def check_hier_selection(q, c1, N1, co, T1, c2, N2, off2, T2, sm, ref, t, label):
    """Masks bit-exact except near-threshold clusters (listed).  Returns rows whose level-1 sets differ."""
    B, H = q.shape[:2]
    C1, C2 = c1.shape[1], c2.shape[1]
    g1 = unpack_mask(t["m1"].cpu().numpy(), C1); g2 = unpack_mask(t["m2"].cpu().numpy(), C2)
    o1 = unpack_mask(ref["mask1"], C1); o2 = unpack_mask(ref["mask2"], C2)
    nk = t["nk"].cpu().numpy()[:, :, 0]; nr = t["nr"].cpu().numpy()[:, :, 0]
    rg = t["ranges"].cpu().numpy()[:, :, 0]
    skipped = []
    for b in range(B):
        for h in range(H):
            l1, l2, S1, S2 = literal.hier_select(q[b, h], c1[h], N1[h], co[h], T1[h], c2[h], N2[h], T2[h], sm)
            d1 = np.flatnonzero(g1[b, h] != o1[b, h])
            assert literal.near_threshold(S1[d1], T1[h]).all(), (label, b, h, "level 1", d1)
            if len(d1):
                print(f"[near-threshold coarse clusters {label}] b{b} h{h}: {d1.tolist()}")
                skipped.append((b, h))
            else:
                d2 = np.flatnonzero(g2[b, h] != o2[b, h])
                assert literal.near_threshold(np.nan_to_num(S2[d2], nan=1.0), T2[h]).all(), (label, b, h, "level 2", d2)
                if len(d2):
                    print(f"[near-threshold fine clusters {label}] b{b} h{h}: {d2.tolist()}")
            # internal consistency of the GPU outputs whatever the oracle says
            cand = np.zeros(C2, bool)
            for j in np.flatnonzero(g1[b, h]):
                cand[co[h, j]:co[h, j + 1]] = True
            assert not (g2[b, h] & ~cand).any()
            ids = np.flatnonzero(g2[b, h])
            assert nr[b, h] == len(ids) and nk[b, h] == N2[h, ids].sum()
            np.testing.assert_array_equal(rg[b, h, :len(ids)], np.stack([off2[h, ids], N2[h, ids]], 1).reshape(-1, 2))
    return g2, skipped


@pytest.mark.parametrize("seed,H,C1,fan", [(0, 2, 6, (1, 5)), (1, 3, 40, (0, 9)), (2, 1, 100, (20, 40)), (3, 2, 33, (64, 64))])
def test_small_hier_select(sq, oracle, seed, H, C1, fan):
    rng = np.random.default_rng(500 + seed)
    q, c1, N1, co, c2, N2, off2 = hier_problem(rng, H, C1, fan[0], fan[1], 128)
    C2 = c2.shape[1]; L = int(off2[:, -1].max())
    q = q.reshape(1, H, 128)
    T1 = np.full(H, 0.6 / N1.sum(1).mean(), np.float32); T2 = np.full(H, 2.0 / N2.sum(1).mean(), np.float32)
    sm = float(np.float32(0.3))
    ref = oracle.hier_select(q, c1, N1, co, T1, c2, N2, off2, T2, sm)
    sh, t = run_hier_select(sq, 1, H, C1, C2, L, q, c1, N1, co, T1, c2, N2, off2, T2, sm)
    check_hier_selection(q, c1, N1, co, T1, c2, N2, off2, T2, sm, ref, t, f"small{seed}")
    assert t["nk"].sum() > 0


def test_hier_select_many_rows(sq, oracle):
    # More than 1024 (sequence, head) rows: the last level's slices are then mapped one workgroup per (row, slice)
    # instead of being dealt over a fixed grid.  Every sequence has its own query; the high threshold at level 1
    # leaves some rows without a single candidate (their counts must still come out as 0).
    rng = np.random.default_rng(77)
    H, C1 = 8, 12
    q1, c1, N1, co, c2, N2, off2 = hier_problem(rng, H, C1, 30, 50, 128)
    C2 = c2.shape[1]; L = int(off2[:, -1].max())
    B = 130                                                   # 1040 rows
    q = (rng.standard_normal((B, H, 128)) * 1.5).astype(np.float16)
    T1 = np.full(H, 3.0 / N1.sum(1).mean(), np.float32); T2 = np.full(H, 2.0 / N2.sum(1).mean(), np.float32)
    sm = float(np.float32(0.3))
    ref = oracle.hier_select(q, c1, N1, co, T1, c2, N2, off2, T2, sm)
    sh, t = run_hier_select(sq, B, H, C1, C2, L, q, c1, N1, co, T1, c2, N2, off2, T2, sm)
    check_hier_selection(q, c1, N1, co, T1, c2, N2, off2, T2, sm, ref, t, "manyrows")
    nk = t["nk"].cpu().numpy()
    assert (nk == 0).any() and (nk > 0).any()


def test_keep_all_coarse_equals_one_level_on_gpu(sq, oracle):
    # T1 < 0 keeps every coarse cluster: the candidates are then all fine clusters in order and level 2 must equal
    # the one-level selection with T2 (same logits, same rule).  The level-2 normaliser is merged from per-item sums,
    # the one-level one is summed in the library's row order: they agree to fp32 rounding (~1e-7 relative), and the
    # calibrated thresholds sit in the middle of a gap between two scores, so no decision can differ here.
    w = wl.make_workload("hier_t1neg", B=2, H=2, L=8192, C=256, Lq=1, U=0, keep_frac=1 / 8, C1=16,
                         coarse_keep_frac=1 / 4, seed=7, threads=2)
    wl.calibrate(w, oracle.scores)
    T1 = np.full(w.H, -1.0, np.float32)
    sh, t = run_hier_select(sq, w.B, w.H, w.C1, w.C, w.L, w.q[:, :, 0], w.centroids1, w.sizes1, w.child_offsets, T1,
                            w.centroids, w.sizes, w.offsets, w.thresh2, w.sm_scale)
    P = sq.upload(w, thresh=w.thresh2)
    sq.sq_centroid_score(P.shape, P.q, P.centroids, P.sizes, P.logits, P.row_max, P.denom)
    sq.sq_select(P.shape, P.logits, P.row_max, P.denom, P.thresh, P.sizes, P.offsets, P.keep_mask, P.ranges,
                 P.n_ranges, P.n_keys)
    torch.cuda.synchronize()
    assert torch.equal(t["m2"], P.keep_mask[:, :, 0]) and torch.equal(t["nk"], P.n_keys)
    assert torch.equal(t["ranges"], P.ranges)


def hier_decode_and_compare(sq, oracle, w, label):
    P = sq.upload(w)
    sh = P.shape
    ws = sq.workspace(sh, sq.SQ_CALL_HIER_DECODE_STEP, P.q.device)
    m2 = torch.zeros(w.B, w.H, (w.C + 31) // 32, dtype=torch.int32, device=P.q.device)
    sq.sq_hier_decode_step(sh, w.C1, P.q, P.centroids1, P.sizes1, P.child_offsets, P.thresh1, P.centroids, P.sizes,
                           P.offsets, P.thresh2, P.K_fixed, P.V_fixed, P.K_user, P.V_user, P.out, P.lse, m2, P.n_keys, ws)
    torch.cuda.synchronize()
    # the separate call must give the same selection as the fused step
    sh2, t = run_hier_select(sq, w.B, w.H, w.C1, w.C, w.L, w.q[:, :, 0], w.centroids1, w.sizes1, w.child_offsets,
                             w.thresh1, w.centroids, w.sizes, w.offsets, w.thresh2, w.sm_scale, U=w.U)
    assert torch.equal(t["m2"], m2) and torch.equal(t["nk"], P.n_keys)
    ref = oracle.hier_select(w.q[:, :, 0], w.centroids1, w.sizes1, w.child_offsets, w.thresh1, w.centroids, w.sizes,
                             w.offsets, w.thresh2, w.sm_scale)
    g2, skipped = check_hier_selection(w.q[:, :, 0], w.centroids1, w.sizes1, w.child_offsets, w.thresh1, w.centroids,
                                       w.sizes, w.offsets, w.thresh2, w.sm_scale, ref, t, label)
    # attention on the GPU's own (validated) selection
    cap = int(g2.sum(-1).max()) + 1
    ranges = np.zeros((w.B, w.H, 1, cap, 2), np.int32); nr = np.zeros((w.B, w.H, 1), np.int32)
    for b in range(w.B):
        for h in range(w.H):
            ranges[b, h, 0], nr[b, h, 0] = ranges_from_keep(g2[b, h], w.offsets[h], w.sizes[h], cap)
    out, lse = oracle.sparse_attn(w.q, w.K_fixed, w.V_fixed, ranges, nr, w.K_user, w.V_user, w.sm_scale)
    err = np.abs(P.out.cpu().numpy().astype(np.float64) - out).max()
    assert err <= ATTN_ATOL, f"{label}: attention max-abs error {err}"
    np.testing.assert_allclose(P.lse.cpu().numpy(), lse, atol=1e-4, rtol=1e-5)
    return P


def test_hier_decode_medium(sq, oracle):
    w = wl.make_workload("hier_medium", B=2, H=4, L=65536, C=2048, Lq=1, U=200, keep_frac=1 / 16, C1=64,
                         coarse_keep_frac=1 / 8, seed=11, threads=4)
    wl.calibrate(w, oracle.scores)
    hier_decode_and_compare(sq, oracle, w, "hier_medium")


def test_cfg5_hier_decode_512k(sq, oracle):
    print("cfg5: generating (8 GiB of K/V)", flush=True)
    w = wl.make_config("cfg5_hier_decode_512k", threads=16)
    print("cfg5: calibrating", flush=True)
    wl.calibrate(w, oracle.scores)
    print("cfg5: running", flush=True)
    P = hier_decode_and_compare(sq, oracle, w, "cfg5")
    nk = P.n_keys.cpu().numpy().ravel()
    print("cfg5 keep fraction per head:", np.round(nk / w.L, 4), "mean", nk.mean() / w.L, flush=True)


@pytest.mark.parametrize("name", ["f3_hier_1pct_prune50_256k", "f3_hier_05pct_prune90_256k"])
def test_paper_hierarchy_sizing_256k(sq, oracle, name):
    """The paper's own sizing of the hierarchy (Section 6 "Experimental Details"; appendix "Hierarchical kernel
    benchmarking"): fine centroids at 5 % of the context, coarse centroids at 1 % / 0.5 %, the first level pruning
    50 % / 90 % of the coarse clusters, variable fan-out; 32 heads x 256K keys through sq_hier_decode_step."""
    print(f"{name}: generating", flush=True)
    w = wl.make_config(name, threads=16)
    print(f"{name}: calibrating", flush=True)
    wl.calibrate(w, oracle.scores)
    fans = np.diff(w.child_offsets, axis=1)
    assert fans.min() >= 1 and fans.max() > fans.min()          # the fan-out does vary
    print(f"{name}: running", flush=True)
    P = hier_decode_and_compare(sq, oracle, w, name)
    nk = P.n_keys.cpu().numpy().ravel()
    print(f"{name}: keep fraction mean {nk.mean() / w.L:.4f} (per head {np.round(nk / w.L, 3).tolist()})", flush=True)
    assert nk.sum() > 0
