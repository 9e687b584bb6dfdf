"""Pins of the two-level lookup with the prefill rule (Appendix D: scores averaged over the query tokens) at both
levels (Section 3.3): a closed form worked by hand, Lq = 1 against the decode-time two-level oracle, a first level
that keeps everything against the one-level averaged selection, and the literal fp64 equations."""
import numpy as np
import pytest

from oracle import literal
from test_oracle_hier import hier_problem
from test_oracle_scores import LN2
from test_oracle_select import unpack


def test_closed_form_two_tokens(oracle):
    # d = 2, sm_scale = ln 2, so every exp() is a power of two.  Token 0 = (1, 0), token 1 = (0, 1).
    # Coarse centroids (3, 0) and (0, 3), two keys under each: token 0 has e = (8, 1), D = 2*8 + 2*1 = 18,
    # S = (8, 1) / 18; token 1 mirrored; the averaged scores are (9/36, 9/36) = (1/4, 1/4): BOTH coarse clusters pass
    # T1 = 0.2 although each token alone would keep only one (1/18 < 0.2), and none passes T1 = 0.26.
    # Fine centroids (4,0), (2,0) under coarse 0 and (0,4), (0,2) under coarse 1, one key each: token 0 has
    # e = (16, 4, 1, 1), D = 22; token 1 (1, 1, 16, 4); averages (17, 5, 17, 5) / 44.
    q = np.array([[[[1, 0], [0, 1]]]], np.float16)
    c1 = np.array([[[3, 0], [0, 3]]], np.float16)
    c2 = np.array([[[4, 0], [2, 0], [0, 4], [0, 2]]], np.float16)
    N1, N2 = np.array([[2, 2]], np.int32), np.array([[1, 1, 1, 1]], np.int32)
    co, off2 = np.array([[0, 2, 4]], np.int32), np.array([[0, 1, 2, 3, 4]], np.int32)
    T = lambda v: np.array([v], np.float32)
    r = oracle.hier_select_mean(q, c1, N1, co, T(0.2), c2, N2, off2, T(0.2), LN2)
    assert r["mask1"][0, 0].tolist() == [True, True]
    assert r["mask2"][0, 0].tolist() == [True, False, True, False]           # 17/44 > 0.2 > 5/44
    assert r["n_keys"][0, 0] == 2 and r["ranges"][0, 0, :2].tolist() == [[0, 1], [2, 1]]
    r = oracle.hier_select_mean(q, c1, N1, co, T(0.2), c2, N2, off2, T(0.1), LN2)
    assert r["mask2"][0, 0].all()
    r = oracle.hier_select_mean(q, c1, N1, co, T(0.26), c2, N2, off2, T(0.1), LN2)
    assert not r["mask1"][0, 0].any() and not r["mask2"][0, 0].any() and r["n_keys"][0, 0] == 0
    k1, k2, S1, S2 = literal.hier_select_mean(q[0, 0], c1[0], N1[0], co[0], 0.2, c2[0], N2[0], 0.2, LN2)
    np.testing.assert_allclose(S1, [0.25, 0.25], rtol=1e-7)
    np.testing.assert_allclose(S2, np.array([17, 5, 17, 5]) / 44, rtol=1e-7)     # (ln 2 is an fp32 constant here)


@pytest.mark.parametrize("seed", range(3))
def test_one_token_is_the_decode_time_lookup(oracle, seed):
    rng = np.random.default_rng(300 + seed)
    q, c1, N1, co, c2, N2, off2 = hier_problem(rng, 3, 9, 1, 6, 32)
    T1 = np.full(3, 0.5 / N1.sum(1).mean(), np.float32)
    T2 = np.full(3, 1.5 / N2.sum(1).mean(), np.float32)
    a = oracle.hier_select(q, c1, N1, co, T1, c2, N2, off2, T2, 0.3)
    b = oracle.hier_select_mean(q[:, :, None, :], c1, N1, co, T1, c2, N2, off2, T2, 0.3)
    np.testing.assert_array_equal(unpack(a["mask1"], 9), b["mask1"])
    np.testing.assert_array_equal(unpack(a["mask2"], c2.shape[1]), b["mask2"])
    np.testing.assert_array_equal(a["n_keys"], b["n_keys"])
    assert b["n_keys"].sum() > 0


def test_first_level_that_keeps_everything_is_the_one_level_averaged_selection(oracle):
    rng = np.random.default_rng(310)
    _, c1, N1, co, c2, N2, off2 = hier_problem(rng, 2, 7, 2, 5, 32, zero_frac=0.0)
    q = rng.standard_normal((2, 2, 6, 32)).astype(np.float16)
    T2 = np.full(2, 1.2 / N2.sum(1).mean(), np.float32)
    r = oracle.hier_select_mean(q, c1, N1, co, np.full(2, -1.0, np.float32), c2, N2, off2, T2, 0.25)
    assert r["mask1"].all()
    x, m, D = oracle.centroid_score(q, c2, N2, 0.25)
    mask, ranges, nr, nk = oracle.select_mean(x, m, D, T2, N2, off2)
    np.testing.assert_array_equal(unpack(mask, c2.shape[1]), r["mask2"])
    np.testing.assert_array_equal(nk, r["n_keys"])
    np.testing.assert_array_equal(ranges, r["ranges"])
    assert 0 < nk.sum() < N2.sum() * 2


@pytest.mark.parametrize("seed", range(3))
def test_against_the_literal_equations(oracle, seed):
    rng = np.random.default_rng(320 + seed)
    _, c1, N1, co, c2, N2, off2 = hier_problem(rng, 2, 10, 0, 7, 32)
    q = (rng.standard_normal((1, 2, 5, 32)) * 0.8).astype(np.float16)
    T1 = np.full(2, 0.6 / N1.sum(1).mean(), np.float32)
    T2 = np.full(2, 1.0 / N2.sum(1).mean(), np.float32)
    r = oracle.hier_select_mean(q, c1, N1, co, T1, c2, N2, off2, T2, 0.3)
    some = 0
    for h in range(2):
        k1, k2, S1, S2 = literal.hier_select_mean(q[0, h], c1[h], N1[h], co[h], T1[h], c2[h], N2[h], T2[h], 0.3)
        d1 = np.flatnonzero(k1 != r["mask1"][0, h])
        assert literal.near_threshold(S1[d1], T1[h]).all()
        if len(d1) == 0:
            d2 = np.flatnonzero(k2 != r["mask2"][0, h])
            assert literal.near_threshold(np.nan_to_num(S2[d2], nan=1.0), T2[h]).all()
        some += int(k2.sum())
        # the averaged fine scores weigh to one over the candidates (Eq. 3 per token, then the mean)
        cand = ~np.isnan(S2)
        if cand.any() and (N2[h][cand] > 0).any():
            assert (S2[cand] * N2[h][cand]).sum() == pytest.approx(1.0, rel=1e-9)
    assert some > 0
