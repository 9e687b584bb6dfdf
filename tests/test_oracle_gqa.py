"""Pins of the grouped-query decode oracle (appendix "Additional Longbench Evaluation": K/V shared amongst a
subset of the heads, every head selects independently).  The oracle walks the query heads one by one; these tests
check it against routes that do not: the one-level oracle on explicitly repeated K/V heads, a dense NumPy softmax
when everything is kept, and the symmetries the definition implies."""
import numpy as np
import pytest

import oracle
from paper_2411_09688_amd import workload as wl
from tests.gpu_util import oracle_one_level, unpack_mask


def make(G, B=2, H=2, L=600, C=24, U=9, keep=0.4, seed=31):
    # Lq = G query rows per (sequence, K/V head) = the G query heads of the group: q [B, H, G, d]
    w = wl.calibrate(wl.make_workload("gqa_oracle", B=B, H=H, L=L, C=C, Lq=G, U=U, keep_frac=keep, seed=seed, threads=1),
                     oracle.scores)
    q = np.ascontiguousarray(w.q.reshape(B, H * G, w.d))       # query head hq = h * G + g
    return w, q


def run(w, q, G, thresh=None):
    return oracle.gqa_decode(q, w.centroids, w.sizes, w.offsets, w.thresh if thresh is None else thresh, w.K_fixed,
                             w.V_fixed, w.K_user, w.V_user, w.sm_scale, G)


@pytest.mark.parametrize("G", [1, 2, 4])
def test_equals_one_level_method_on_repeated_kv_heads(G):
    w, q = make(G)
    got = run(w, q, G)
    rep = lambda a, ax=0: np.repeat(a, G, axis=ax)
    x, m, D = oracle.centroid_score(q[:, :, None, :], rep(w.centroids), rep(w.sizes), w.sm_scale)
    mask, ranges, n_r, n_k = oracle.select(x, m, D, rep(w.thresh), rep(w.sizes), rep(w.offsets))
    out, lse = oracle.sparse_attn(q[:, :, None, :], rep(w.K_fixed), rep(w.V_fixed), ranges, n_r, rep(w.K_user, 1),
                                  rep(w.V_user, 1), w.sm_scale)
    np.testing.assert_array_equal(got["mask"], mask[:, :, 0])
    np.testing.assert_array_equal(got["n_keys"], n_k[:, :, 0])
    np.testing.assert_array_equal(got["out"], out[:, :, 0])
    np.testing.assert_array_equal(got["lse"], lse[:, :, 0])
    assert 0 < got["n_keys"].mean() < w.L                       # a real selection took place


def test_group_of_one_is_the_plain_decode_step():
    w, q = make(1)
    got = run(w, q, 1)
    ref = oracle_one_level(oracle, w)
    out, lse = oracle.sparse_attn(w.q, w.K_fixed, w.V_fixed, ref["ranges"], ref["n_ranges"], w.K_user, w.V_user, w.sm_scale)
    np.testing.assert_array_equal(got["mask"], ref["mask"][:, :, 0])
    np.testing.assert_array_equal(got["out"], out[:, :, 0])


def test_keep_all_is_dense_attention_over_the_shared_kv_head():
    G = 4
    w, q = make(G, B=1, H=2, L=300, C=10, U=7)
    got = run(w, q, G, thresh=np.full(w.H, -1.0, np.float32))
    assert (got["n_keys"] == w.L).all()
    for hq in range(w.H * G):
        h = hq // G
        K = np.concatenate([w.K_fixed[h], w.K_user[0, h]]).astype(np.float64)
        V = np.concatenate([w.V_fixed[h], w.V_user[0, h]]).astype(np.float64)
        s = np.float64(w.sm_scale) * (K @ q[0, hq].astype(np.float64))
        p = np.exp(s - s.max())
        np.testing.assert_allclose(got["out"][0, hq], (p[:, None] * V).sum(0) / p.sum(), rtol=0, atol=1e-12)
        np.testing.assert_allclose(got["lse"][0, hq], s.max() + np.log(p.sum()), rtol=0, atol=1e-12)


def test_heads_of_a_group_are_independent_and_share_only_the_kv_head():
    G = 2
    w, q = make(G)
    base = run(w, q, G)
    # identical queries in a group -> identical results
    q2 = q.copy()
    q2[:, 1] = q2[:, 0]
    same = run(w, q2, G)
    np.testing.assert_array_equal(same["out"][:, 0], same["out"][:, 1])
    np.testing.assert_array_equal(same["mask"][:, 0], same["mask"][:, 1])
    # changing one head's query leaves the other heads untouched
    np.testing.assert_array_equal(same["out"][:, 0], base["out"][:, 0])
    np.testing.assert_array_equal(same["out"][:, 2:], base["out"][:, 2:])
    # a query moved to the other K/V head meets different keys
    q3 = q.copy()
    q3[:, 2] = q[:, 0]
    other = run(w, q3, G)
    assert np.abs(other["out"][:, 2] - base["out"][:, 0]).max() > 1e-3
    # selections of the two heads of a group differ (each head selects on its own)
    keep = unpack_mask(base["mask"], w.C)
    assert (keep[:, 0] != keep[:, 1]).any()


# ---- one kept set per K/V head from scores averaged over the group --------------------------------------------------

def test_group_average_keeps_what_no_single_head_would():
    # Two query heads on one K/V head, d = 2, sm_scale = ln 2: head 0 = (1, 0), head 1 = (0, 1); clusters with
    # centroids (3, 0) and (0, 3), two keys each.  Head 0 alone: e = (8, 1), D = 18, S = (8/18, 1/18); head 1 mirrored.
    # With T = 0.2 each head on its own keeps ONE cluster; the group average (1/4, 1/4) keeps BOTH.
    import oracle
    LN2 = float(np.log(2.0))
    q = np.array([[[1, 0], [0, 1]]], np.float16)                 # [B = 1, Hq = 2, d]
    cent = np.array([[[3, 0], [0, 3]]], np.float16)
    sizes, offsets = np.array([[2, 2]], np.int32), np.array([[0, 2, 4]], np.int32)
    K = np.array([[[3, 0], [3, 0], [0, 3], [0, 3]]], np.float16)
    V = np.array([[[1, 0], [1, 0], [0, 1], [0, 1]]], np.float16)
    Ku = np.zeros((1, 1, 0, 2), np.float16)
    T = np.array([0.2], np.float32)
    own = oracle.gqa_decode(q, cent, sizes, offsets, T, K, V, Ku, Ku, LN2, 2)
    assert own["n_keys"].tolist() == [[2, 2]] and own["mask"][0, :, 0].tolist() == [1, 2]
    avg = oracle.gqa_mean_decode(q, cent, sizes, offsets, T, K, V, Ku, Ku, LN2, 2)
    assert avg["n_keys"].tolist() == [[4]] and avg["mask"][0, 0, 0] == 3
    # head 0 over all four keys: weights (8, 8, 1, 1) / 18 on values (1,0), (1,0), (0,1), (0,1)
    np.testing.assert_allclose(avg["out"][0, 0], [16 / 18, 2 / 18], rtol=1e-6)
    np.testing.assert_allclose(avg["out"][0, 1], [2 / 18, 16 / 18], rtol=1e-6)
    np.testing.assert_allclose(avg["lse"][0], [np.log(18.0)] * 2, rtol=1e-6)


def test_group_of_one_average_is_the_plain_step():
    import oracle
    rng = np.random.default_rng(77)
    H, C, L, U, d = 3, 20, 200, 7, 128
    cent = (rng.standard_normal((H, C, d)) * 0.6).astype(np.float16)
    sizes = rng.multinomial(L, np.full(C, 1 / C), size=H).astype(np.int32)
    offsets = np.zeros((H, C + 1), np.int32); offsets[:, 1:] = np.cumsum(sizes, 1)
    K = rng.standard_normal((H, L, d)).astype(np.float16); V = rng.standard_normal((H, L, d)).astype(np.float16)
    Ku = rng.standard_normal((2, H, U, d)).astype(np.float16); Vu = rng.standard_normal((2, H, U, d)).astype(np.float16)
    q = rng.standard_normal((2, H, d)).astype(np.float16)
    T = np.full(H, 1.0 / L, np.float32)
    a = oracle.gqa_decode(q, cent, sizes, offsets, T, K, V, Ku, Vu, 0.3, 1)
    b = oracle.gqa_mean_decode(q, cent, sizes, offsets, T, K, V, Ku, Vu, 0.3, 1)
    np.testing.assert_array_equal(a["mask"], b["mask"])
    np.testing.assert_array_equal(a["n_keys"], b["n_keys"])
    np.testing.assert_allclose(a["out"], b["out"], rtol=0, atol=1e-12)
    assert 0 < b["n_keys"].sum() < 2 * H * L
