"""Pins of the oracle's lookup through any number of centroid levels (Section 3.3 applied level after level).
Checked against the two-level oracle (n = 2), the one-level selection (n = 1), the collapse of a level that keeps
everything, the literal fp64 equations, and the normalisation of every level over its candidates only."""
import numpy as np
import pytest

from oracle import literal
from test_oracle_hier import hier_problem
from test_oracle_select import unpack


def three_level_problem(rng, H, C0, fan01, fan12, d):
    """Levels 0 -> 1 -> 2: level-2 clusters hold keys; a coarser centroid is the mean of its children's centroids and
    its size the number of keys underneath."""
    q, c1, N1, co1, c2, N2, off2 = hier_problem(rng, H, C0 * fan01, fan12[0], fan12[1], d)
    C1 = c1.shape[1]
    co0 = np.tile(np.arange(C0 + 1, dtype=np.int32) * fan01, (H, 1))
    c0 = c1.astype(np.float64).reshape(H, C0, fan01, d).mean(axis=2).astype(np.float16)
    N0 = N1.reshape(H, C0, fan01).sum(axis=2).astype(np.int32)
    lv = lambda c, n, co, T: dict(centroids=c, sizes=n, child_offsets=co, thresh=np.full(H, T, np.float32))
    return q, [lv(c0, N0, co0, 0.0), lv(c1, N1, co1, 0.0), lv(c2, N2, off2, 0.0)]


def with_thresholds(levels, Ts):
    return [dict(l, thresh=np.full_like(l["thresh"], T)) for l, T in zip(levels, Ts)]


@pytest.mark.parametrize("seed", range(3))
def test_two_levels_equal_the_two_level_oracle(oracle, seed):
    rng = np.random.default_rng(500 + seed)
    H = 3
    q, c1, N1, co, c2, N2, off2 = hier_problem(rng, H, 9, 0, 6, 64)
    T1 = np.full(H, 0.012, np.float32); T2 = np.full(H, 0.03, np.float32)
    ref = oracle.hier_select(q, c1, N1, co, T1, c2, N2, off2, T2, 0.3)
    got = oracle.multilevel_select(q[0][None], [dict(centroids=c1, sizes=N1, child_offsets=co, thresh=T1),
                                               dict(centroids=c2, sizes=N2, child_offsets=off2, thresh=T2)], 0.3)
    np.testing.assert_array_equal(got["masks"][0], ref["mask1"])
    np.testing.assert_array_equal(got["masks"][1], ref["mask2"])
    np.testing.assert_array_equal(got["ranges"], ref["ranges"])
    np.testing.assert_array_equal(got["n_keys"], ref["n_keys"])
    assert 0 < got["n_keys"].sum() < N2.sum()


def test_one_level_equals_plain_selection(oracle):
    rng = np.random.default_rng(510)
    H = 2
    q, c1, N1, co, c2, N2, off2 = hier_problem(rng, H, 5, 2, 6, 32)
    T = np.full(H, 0.02, np.float32)
    got = oracle.multilevel_select(q[0][None], [dict(centroids=c2, sizes=N2, child_offsets=off2, thresh=T)], 0.3)
    x, m, D = oracle.centroid_score(q[:, :, None], c2, N2, 0.3)
    mask, ranges, nr, nk = oracle.select(x, m, D, T, N2, off2)
    np.testing.assert_array_equal(got["masks"][0], mask[:, :, 0])
    np.testing.assert_array_equal(got["ranges"], ranges[:, :, 0])
    np.testing.assert_array_equal(got["n_keys"], nk[:, :, 0])


@pytest.mark.parametrize("seed", range(3))
def test_a_level_that_keeps_everything_drops_out(oracle, seed):
    rng = np.random.default_rng(520 + seed)
    H = 2
    q, levels = three_level_problem(rng, H, 4, 3, (1, 5), 32)
    q1 = q[0][None]
    # level 0 keeps all: the three-level lookup is the two-level lookup on levels 1, 2
    a = oracle.multilevel_select(q1, with_thresholds(levels, (-1.0, 0.01, 0.03)), 0.3)
    b = oracle.multilevel_select(q1, with_thresholds(levels[1:], (0.01, 0.03)), 0.3)
    # (level-1 clusters under an empty level-0 cluster are empty themselves)
    np.testing.assert_array_equal(a["masks"][2], b["masks"][1])
    np.testing.assert_array_equal(a["ranges"], b["ranges"])
    # levels 0 and 1 keep all: one-level selection on the finest level
    c = oracle.multilevel_select(q1, with_thresholds(levels, (-1.0, -1.0, 0.009)), 0.3)
    e = oracle.multilevel_select(q1, with_thresholds(levels[2:], (0.009,)), 0.3)
    np.testing.assert_array_equal(c["masks"][2], e["masks"][0])
    np.testing.assert_array_equal(c["n_keys"], e["n_keys"])
    assert a["n_keys"].sum() > 0 and c["n_keys"].sum() > 0


@pytest.mark.parametrize("seed", range(4))
def test_three_levels_structure_and_bruteforce(oracle, seed):
    rng = np.random.default_rng(530 + seed)
    H = 3
    q, levels = three_level_problem(rng, H, 5, 2, (0, 5), 64)
    Ts = (0.004, 0.012, 0.03)
    levels = with_thresholds(levels, Ts)
    got = oracle.multilevel_select(q[0][None], levels, 0.3)
    kept_any = 0
    for h in range(H):
        lit = literal.multilevel_select(q[0, h], [(l["centroids"][h], l["sizes"][h], l["child_offsets"][h], l["thresh"][h])
                                                  for l in levels], 0.3)
        agree = True
        for k, l in enumerate(levels):
            Ck = l["centroids"].shape[1]
            keep = unpack(got["masks"][k], Ck)[0, h]
            lk, S = lit[k]
            cand = ~np.isnan(S)
            if agree:
                # Eq. 3: every level's scores are normalised over its own candidates only
                if cand.any() and l["sizes"][h][cand].sum() > 0:
                    assert (S[cand] * l["sizes"][h][cand]).sum() == pytest.approx(1.0, rel=1e-12)
                near = literal.near_threshold(np.nan_to_num(S, nan=1.0), l["thresh"][h])
                assert not ((keep != lk) & ~near).any(), (h, k)
                assert not (keep & ~cand).any()                # kept clusters are children of kept parents
                agree = (keep == lk).all()
        last = unpack(got["masks"][-1], levels[-1]["centroids"].shape[1])[0, h]
        assert got["n_keys"][0, h] == levels[-1]["sizes"][h][last].sum()
        assert got["n_ranges"][0, h] == last.sum()
        ids = np.flatnonzero(last)
        np.testing.assert_array_equal(got["ranges"][0, h, :len(ids), 0], levels[-1]["child_offsets"][h][ids])
        np.testing.assert_array_equal(got["ranges"][0, h, :len(ids), 1], levels[-1]["sizes"][h][ids])
        kept_any += last.sum()
    assert kept_any > 0
