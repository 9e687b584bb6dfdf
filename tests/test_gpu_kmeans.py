"""GPU parity: offline clustering (Section 3.1) through the C ABI against the NumPy oracle.

What is unique is compared exactly: the assignment wherever the two best centres are more than MARGIN apart in
score (closer pairs may go either way in fp32 and must still be a best centre within MARGIN), and -- from the
GPU's own assignment -- sizes, offsets and the stable grouping, bit for bit.  Centres are fp16 roundings of
fp32 / fp64 means: at most one fp16 unit apart."""
import numpy as np
import pytest
import torch

from gpu_util import unpack_mask
from oracle import clustering as ocl
from paper_2411_09688_amd import workload as wl

pytestmark = pytest.mark.gpu

MARGIN = 1e-5          # score gap below which fp32 and fp64 may order two centres differently (|x|, |c| <= 1)
DEV = "cuda:0"
UNIT_ATOL = 5e-4       # one fp16 unit for magnitudes below 1 (normalised vectors and their means)


@pytest.fixture(scope="module")
def sq():
    from paper_2411_09688_amd import binding
    binding.lib()
    return binding


def t(a, dtype=None):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV, dtype=dtype)


def gpu_step(sq, X, cent):
    """One sq_kmeans_step on X [H, L, d], cent [H, C, d] (numpy f16) -> numpy outputs."""
    H, L, d = X.shape
    C = cent.shape[1]
    sh = sq.make_shape(1, H, L, C, 1, 0, 1.0)
    Xg, cg = t(X), t(cent)
    out = torch.full_like(cg, 7.0)
    assign = torch.full((H, L), -1, dtype=torch.int32, device=DEV)
    sizes = torch.full((H, C), -1, dtype=torch.int32, device=DEV)
    offsets = torch.full((H, C + 1), -1, dtype=torch.int32, device=DEV)
    perm = torch.full((H, L), -1, dtype=torch.int32, device=DEV)
    ws = sq.workspace(sh, sq.SQ_CALL_KMEANS_STEP, DEV)
    sq.sq_kmeans_step(sh, Xg, cg, out, assign, sizes, offsets, perm, ws)
    torch.cuda.synchronize()
    return [x.cpu().numpy() for x in (assign, sizes, offsets, perm, out)]


def check_step(X, cent, got, label):
    assign, sizes, offsets, perm, cent_new = got
    H, L, _ = X.shape
    C = cent.shape[1]
    close = 0
    for h in range(H):
        a_ref, margin = ocl.assign(X[h], cent[h])
        clear = margin > MARGIN
        np.testing.assert_array_equal(assign[h][clear], a_ref[clear], err_msg=f"{label} head {h}")
        amb = np.flatnonzero(~clear)
        close += len(amb)
        if len(amb):
            Xd, Cd = X[h][amb].astype(np.float64), cent[h].astype(np.float64)
            s = Xd @ Cd.T - 0.5 * (Cd * Cd).sum(1)[None, :]
            chosen = s[np.arange(len(amb)), assign[h][amb]]
            assert (s.max(1) - chosen <= MARGIN).all(), f"{label} head {h}: a near-tie went to a centre that is not best"
        assert assign[h].min() >= 0 and assign[h].max() < C
        # bookkeeping of the GPU's own assignment: exact
        np.testing.assert_array_equal(sizes[h], np.bincount(assign[h], minlength=C))
        np.testing.assert_array_equal(offsets[h], np.concatenate([[0], np.cumsum(sizes[h])]))
        np.testing.assert_array_equal(perm[h], np.argsort(assign[h], kind="stable"))
        c_ref, _ = ocl.update(X[h], assign[h], cent[h])
        err = np.abs(cent_new[h].astype(np.float64) - c_ref.astype(np.float64)).max()
        assert err <= UNIT_ATOL, f"{label} head {h}: centre error {err}"
        empty = sizes[h] == 0
        np.testing.assert_array_equal(cent_new[h][empty], cent[h][empty])      # a centre without members keeps its value
    return close


@pytest.mark.parametrize("H,L,C,mix", [
    (2, 3000, 70, 0),          # ragged: L not a multiple of the 128-key tile, C not a multiple of the 64-centre group
    (1, 4097, 130, 40),        # more centres than generating clusters: many near-equal scores
    (3, 640, 64, 0),           # exactly one group of centres
    (1, 70000, 300, 0),        # 55 parts per head in the grouping
    (1, 129, 129, 0),          # every key its own centre
    (1, 1, 1, 0),              # the smallest problem
    (2, 100, 1, 3),            # one centre takes everything
])
def test_one_iteration_matches_the_oracle(sq, H, L, C, mix):
    K, _, init = wl.clustering_input(11, H, L, C, mix=mix)
    X = np.stack([ocl.normalize_rows(K[h]) for h in range(H)])
    cent = np.stack([X[h][init[h]] for h in range(H)])
    got = gpu_step(sq, X, cent)
    check_step(X, cent, got, f"H{H} L{L} C{C}")


def test_normalisation(sq):
    K, _, _ = wl.clustering_input(12, 2, 1000, 8)
    K[0, 5] = 0                                                  # a zero row stays zero
    sh = sq.make_shape(1, 2, 1000, 8, 1, 0, 1.0)
    Kg = t(K)
    Xg = torch.empty_like(Kg)
    sq.sq_kmeans_normalize(sh, Kg, Xg)
    torch.cuda.synchronize()
    ref = np.stack([ocl.normalize_rows(K[h]) for h in range(2)])
    got = Xg.cpu().numpy()
    assert np.abs(got.astype(np.float64) - ref.astype(np.float64)).max() <= UNIT_ATOL
    assert (got[0, 5] == 0).all()


def test_duplicate_and_far_centres_stay_empty_and_keep_their_value(sq):
    K, _, init = wl.clustering_input(13, 1, 2000, 20)
    X = np.stack([ocl.normalize_rows(K[0])])
    cent = X[:, init[0]].copy()
    cent[0, 7] = cent[0, 3]                                      # a duplicate: equal scores go to the lower index
    cent[0, 11] = (-4 * X[0].astype(np.float32).mean(0)).astype(np.float16) + np.float16(3.0)   # far from every key
    got = gpu_step(sq, X, cent)
    check_step(X, cent, got, "empty")
    sizes = got[1]
    assert sizes[0, 7] == 0 and sizes[0, 11] == 0


def test_lloyd_iterations_track_the_oracle_and_lower_the_objective(sq):
    H, L, C = 2, 6000, 96
    K, _, init = wl.clustering_input(14, H, L, C)
    X = np.stack([ocl.normalize_rows(K[h]) for h in range(H)])
    cent = np.stack([X[h][init[h]] for h in range(H)])
    objs = []
    for it in range(6):
        got = gpu_step(sq, X, cent)
        check_step(X, cent, got, f"iteration {it}")
        a = got[0]
        objs.append(sum(float(((X[h].astype(np.float64) - cent[h].astype(np.float64)[a[h]]) ** 2).sum()) for h in range(H)))
        cent = got[4]                                            # the next iteration starts from the GPU's centres
    assert all(b <= a * (1 + 1e-3) for a, b in zip(objs, objs[1:])), objs
    assert objs[-1] < 0.9 * objs[0]


def test_in_place_centres(sq):
    K, _, init = wl.clustering_input(15, 1, 3000, 50)
    X = np.stack([ocl.normalize_rows(K[0])])
    cent = X[:, init[0]].copy()
    ref = gpu_step(sq, X, cent)
    sh = sq.make_shape(1, 1, 3000, 50, 1, 0, 1.0)
    Xg, cg = t(X), t(cent)
    i32 = lambda *s: torch.empty(s, dtype=torch.int32, device=DEV)
    a, n, o, p = i32(1, 3000), i32(1, 50), i32(1, 51), i32(1, 3000)
    sq.sq_kmeans_step(sh, Xg, cg, cg, a, n, o, p, sq.workspace(sh, sq.SQ_CALL_KMEANS_STEP, DEV))
    torch.cuda.synchronize()
    np.testing.assert_array_equal(cg.cpu().numpy(), ref[4])
    np.testing.assert_array_equal(a.cpu().numpy(), ref[0])


def test_layout_feeds_the_online_path(sq, oracle):
    """Cluster on the GPU, lay the keys out, and run a decode step on the result: the reordered keys are exactly the
    permuted input, the centroids the raw-key means, and the step agrees with the oracle on the same layout."""
    H, L, C, U = 2, 4000, 80, 64
    K, V, init = wl.clustering_input(16, H, L, C)
    sh = sq.make_shape(1, H, L, C, 1, U, 1.0 / np.sqrt(128))
    Kg, Vg = t(K), t(V)
    Xg = torch.empty_like(Kg)
    sq.sq_kmeans_normalize(sh, Kg, Xg)
    cg = torch.stack([Xg[h][t(init[h]).long()] for h in range(H)]).contiguous()
    i32 = lambda *s: torch.empty(s, dtype=torch.int32, device=DEV)
    a, n, o, p = i32(H, L), i32(H, C), i32(H, C + 1), i32(H, L)
    ws = sq.workspace(sh, sq.SQ_CALL_KMEANS_STEP, DEV)
    for _ in range(4):
        sq.sq_kmeans_step(sh, Xg, cg, cg, a, n, o, p, ws)
    Ks, Vs = torch.empty_like(Kg), torch.empty_like(Vg)
    cent = torch.empty(H, C, 128, dtype=torch.float16, device=DEV)
    sq.sq_cluster_layout(sh, Kg, Vg, p, n, o, Ks, Vs, cent)
    torch.cuda.synchronize()
    an, pn, nn, on = a.cpu().numpy(), p.cpu().numpy(), n.cpu().numpy(), o.cpu().numpy()
    for h in range(H):
        perm, sizes, offsets, c_ref = ocl.layout(K[h], an[h], C)
        np.testing.assert_array_equal(pn[h], perm)
        np.testing.assert_array_equal(nn[h], sizes)
        np.testing.assert_array_equal(on[h], offsets)
        np.testing.assert_array_equal(Ks[h].cpu().numpy(), K[h][perm])
        np.testing.assert_array_equal(Vs[h].cpu().numpy(), V[h][perm])
        np.testing.assert_allclose(cent[h].cpu().numpy().astype(np.float64), c_ref.astype(np.float64), rtol=1.1e-3, atol=1e-6)
    # a decode step on the GPU-made layout against the oracle on the same arrays
    rng = np.random.default_rng(160)
    q = (cent.cpu().numpy()[:, 5][None, :, None, :] + 0.3 * rng.standard_normal((1, H, 1, 128))).astype(np.float16)
    Ku = rng.standard_normal((1, H, U, 128)).astype(np.float16)
    Vu = rng.standard_normal((1, H, U, 128)).astype(np.float16)
    cn = cent.cpu().numpy()
    S = np.stack([oracle.scores(q[0, h], cn[h], nn[h], float(sh.sm_scale))[0] for h in range(H)])
    thresh = np.empty(H, np.float32)
    for h in range(H):                                           # between two well-separated scores, about a quarter kept
        srt = np.sort(S[h][nn[h] > 0])[::-1]
        k = next(i for i in range(len(srt) // 4, len(srt) - 1) if srt[i] > 1.01 * srt[i + 1])
        thresh[h] = np.sqrt(srt[k] * srt[k + 1])
    out = torch.empty(1, H, 1, 128, dtype=torch.float16, device=DEV)
    lse = torch.empty(1, H, 1, dtype=torch.float32, device=DEV)
    mask = torch.zeros(1, H, 1, (C + 31) // 32, dtype=torch.int32, device=DEV)
    nk = torch.zeros(1, H, 1, dtype=torch.int32, device=DEV)
    sq.sq_decode_step(sh, t(q), cent, n, o, t(thresh), Ks, Vs, t(Ku), t(Vu), out, lse, mask, nk,
                      sq.workspace(sh, sq.SQ_CALL_DECODE_STEP, DEV))
    torch.cuda.synchronize()
    x, m, Dn = oracle.centroid_score(q, cn, nn, float(sh.sm_scale))
    rmask, ranges, nr, rnk = oracle.select(x, m, Dn, thresh, nn, on)
    ro, _ = oracle.sparse_attn(q, Ks.cpu().numpy(), Vs.cpu().numpy(), ranges, nr, Ku, Vu, float(sh.sm_scale))
    assert 0 < int(nk.sum()) < H * L
    np.testing.assert_array_equal(unpack_mask(mask.cpu().numpy(), C), unpack_mask(rmask, C))
    np.testing.assert_array_equal(nk.cpu().numpy(), rnk)
    assert np.abs(out.cpu().numpy().astype(np.float64) - ro).max() <= 2e-3


def test_full_size_iteration_on_sampled_keys_and_centres(sq):
    """The shape the benchmark times (32 heads x 32768 keys x 1024 centres), in the same launch configuration: sampled
    keys against the oracle's assignment, whole-array properties of the grouping, sampled centres against their
    members' means."""
    cfg = wl.KMEANS_CONFIGS["kmeans_32k"]
    H, L, C = cfg["H"], cfg["L"], cfg["C"]
    K, _, init = wl.clustering_input(0, H, L, C)
    sh = sq.make_shape(1, H, L, C, 1, 0, 1.0)
    Kg = t(K)
    Xg = torch.empty_like(Kg)
    sq.sq_kmeans_normalize(sh, Kg, Xg)
    cg = torch.stack([Xg[h][t(init[h]).long()] for h in range(H)]).contiguous()
    out = torch.empty_like(cg)
    i32 = lambda *s: torch.empty(s, dtype=torch.int32, device=DEV)
    a, n, o, p = i32(H, L), i32(H, C), i32(H, C + 1), i32(H, L)
    sq.sq_kmeans_step(sh, Xg, cg, out, a, n, o, p, sq.workspace(sh, sq.SQ_CALL_KMEANS_STEP, DEV))
    torch.cuda.synchronize()
    X, cent, an, nn, on, pn, cn = (x.cpu().numpy() for x in (Xg, cg, a, n, o, p, out))
    rng = np.random.default_rng(5)
    for h in range(H):
        ks = rng.integers(0, L, 64)
        ks[:2] = (0, L - 1)
        a_ref, margin = ocl.assign(X[h][ks], cent[h])
        clear = margin > MARGIN
        np.testing.assert_array_equal(an[h][ks][clear], a_ref[clear], err_msg=f"head {h}")
        assert clear.mean() > 0.9
        # grouping: exact bookkeeping of the whole head
        np.testing.assert_array_equal(nn[h], np.bincount(an[h], minlength=C))
        np.testing.assert_array_equal(on[h], np.concatenate([[0], np.cumsum(nn[h])]))
        np.testing.assert_array_equal(pn[h], np.argsort(an[h], kind="stable"))
        for c in rng.integers(0, C, 8):
            mem = pn[h][on[h][c]:on[h][c + 1]]
            ref = X[h][mem].astype(np.float64).mean(0) if len(mem) else cent[h][c].astype(np.float64)
            assert np.abs(cn[h][c].astype(np.float64) - ref).max() <= UNIT_ATOL


@pytest.mark.parametrize("H,L,C2,C1,U,mix", [
    (2, 12000, 160, 12, 40, 48),
    (2, 32768, 1638, 328, 128, 400),       # the paper's sizing: fine centroids 5 % of the keys, coarse 1 %
])
def test_two_level_hierarchy_built_on_the_gpu_feeds_the_hierarchical_lookup(sq, oracle, H, L, C2, C1, U, mix):
    """Keys -> fine K-means -> K-means of the fine centroids -> nesting -> layouts, all through the C ABI; every array
    against the oracle's composition of the same steps, then sq_hier_decode_step on the result against the oracle's
    two-level lookup and sparse attention on the same arrays."""
    from test_gpu_hier import check_hier_selection
    from gpu_util import ranges_from_keep
    K, V, init = wl.clustering_input(21, H, L, C2, mix=mix)
    _, _, init1 = wl.clustering_input(22, H, C2, C1)             # (only the seeding indices are used)
    i32 = lambda *s: torch.empty(s, dtype=torch.int32, device=DEV)
    f16 = lambda *s: torch.empty(s, dtype=torch.float16, device=DEV)
    sh = sq.make_shape(1, H, L, C2, 1, U, 1.0 / np.sqrt(128))
    ws = sq.workspace(sh, sq.SQ_CALL_KMEANS_STEP, DEV)
    Kg, Vg = t(K), t(V)
    Xg = torch.empty_like(Kg)
    sq.sq_kmeans_normalize(sh, Kg, Xg)
    cg = torch.stack([Xg[h][t(init[h]).long()] for h in range(H)]).contiguous()
    a2, n2, o2, p2 = i32(H, L), i32(H, C2), i32(H, C2 + 1), i32(H, L)
    for _ in range(3):
        sq.sq_kmeans_step(sh, Xg, cg, cg, a2, n2, o2, p2, ws)
    cent2_old = f16(H, C2, 128)
    sq.sq_cluster_layout(sh, Kg, None, p2, n2, o2, None, None, cent2_old)
    # coarse level: K-means of the (normalised) fine centroids
    shc = sq.make_shape(1, H, C2, C1, 1, 0, 1.0)
    wsc = sq.workspace(shc, sq.SQ_CALL_KMEANS_STEP, DEV)
    X2 = torch.empty_like(cent2_old)
    sq.sq_kmeans_normalize(shc, cent2_old, X2)
    c1g = torch.stack([X2[h][t(init1[h]).long()] for h in range(H)]).contiguous()
    a1, fan, co, p1 = i32(H, C2), i32(H, C1), i32(H, C1 + 1), i32(H, C2)
    for _ in range(3):
        sq.sq_kmeans_step(shc, X2, c1g, c1g, a1, fan, co, p1, wsc)
    # nesting and layouts
    an, n2n, o2n, p2n, n1 = i32(H, L), i32(H, C2), i32(H, C2 + 1), i32(H, L), i32(H, C1)
    sq.sq_cluster_nest(sh, C1, a2, p1, co, an, n2n, o2n, p2n, n1, ws)
    Ks, Vs, cent2 = torch.empty_like(Kg), torch.empty_like(Vg), f16(H, C2, 128)
    sq.sq_cluster_layout(sh, Kg, Vg, p2n, n2n, o2n, Ks, Vs, cent2)
    cent1 = f16(H, C1, 128)
    sq.sq_cluster_layout(shc, cent2, None, None, fan, co, None, None, cent1)
    torch.cuda.synchronize()
    g = {k: v.cpu().numpy() for k, v in dict(a2=a2, a1=a1, p1=p1, co=co, fan=fan, an=an, n2=n2n, o2=o2n, p2=p2n, n1=n1,
                                             Ks=Ks, Vs=Vs, c2=cent2, c1=cent1).items()}
    for h in range(H):
        an_ref, n2_ref, o2_ref, p2_ref, n1_ref = ocl.nest(g["a2"][h], g["p1"][h], g["co"][h], C2)
        for name, ref in (("an", an_ref), ("n2", n2_ref), ("o2", o2_ref), ("p2", p2_ref), ("n1", n1_ref)):
            np.testing.assert_array_equal(g[name][h], ref, err_msg=f"{name} head {h}")
        np.testing.assert_array_equal(g["Ks"][h], K[h][p2_ref])
        np.testing.assert_array_equal(g["Vs"][h], V[h][p2_ref])
        _, _, _, c2_ref = ocl.layout(K[h], an_ref, C2)
        np.testing.assert_allclose(g["c2"][h].astype(np.float64), c2_ref.astype(np.float64), rtol=1.1e-3, atol=1e-6)
        for j in range(C1):                                      # coarse centroid = unweighted mean of its children
            ch = g["c2"][h][g["co"][h][j]:g["co"][h][j + 1]].astype(np.float64)
            ref = ch.mean(0) if len(ch) else np.zeros(128)
            np.testing.assert_allclose(g["c1"][h][j].astype(np.float64), ref, rtol=1.1e-3, atol=1e-6)
        assert g["n1"][h].sum() == L and (np.diff(g["co"][h]) == g["fan"][h]).all()
    # the hierarchical decode step on the GPU-made arrays
    rng = np.random.default_rng(23)
    pick = rng.integers(0, C2, H)
    q = (np.stack([g["c2"][h][pick[h]] for h in range(H)])[None, :, None, :].astype(np.float32)
         + 0.3 * rng.standard_normal((1, H, 1, 128))).astype(np.float16)
    Ku = rng.standard_normal((1, H, U, 128)).astype(np.float16)
    Vu = rng.standard_normal((1, H, U, 128)).astype(np.float16)
    T1 = np.full(H, 0.5 / L, np.float32)
    T2 = np.full(H, 1.0 / L, np.float32)
    sm = float(sh.sm_scale)
    out, lse = f16(1, H, 1, 128), torch.empty(1, H, 1, dtype=torch.float32, device=DEV)
    m2, nk = torch.zeros(1, H, (C2 + 31) // 32, dtype=torch.int32, device=DEV), i32(1, H, 1)
    sq.sq_hier_decode_step(sh, C1, t(q), cent1, n1, co, t(T1), cent2, n2n, o2n, t(T2), Ks, Vs, t(Ku), t(Vu), out, lse,
                           m2, nk, sq.workspace(sh, sq.SQ_CALL_HIER_DECODE_STEP, DEV))
    from test_gpu_hier import run_hier_select
    _, tt = run_hier_select(sq, 1, H, C1, C2, L, q[:, :, 0], g["c1"], g["n1"], g["co"], T1, g["c2"], g["n2"], g["o2"], T2,
                            sm, U=U)
    assert torch.equal(tt["m2"], m2) and torch.equal(tt["nk"], nk)
    ref = oracle.hier_select(q[:, :, 0], g["c1"], g["n1"], g["co"], T1, g["c2"], g["n2"], g["o2"], T2, sm)
    g2, _ = check_hier_selection(q[:, :, 0], g["c1"], g["n1"], g["co"], T1, g["c2"], g["n2"], g["o2"], T2, sm, ref, tt,
                                 "gpu-built hierarchy")
    assert 0 < int(nk.sum()) < H * L
    cap = int(g2.sum(-1).max()) + 1
    ranges = np.zeros((1, H, 1, cap, 2), np.int32)
    nr = np.zeros((1, H, 1), np.int32)
    for h in range(H):
        ranges[0, h, 0], nr[0, h, 0] = ranges_from_keep(g2[0, h], g["o2"][h], g["n2"][h], cap)
    ro, _ = oracle.sparse_attn(q, g["Ks"], g["Vs"], ranges, nr, Ku, Vu, sm)
    assert np.abs(out.cpu().numpy().astype(np.float64) - ro).max() <= 2e-3
