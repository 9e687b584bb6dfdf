"""Pins for the oracle's two-level lookup (Eq. 2-3, Section 3.3)."""
import numpy as np
import pytest

from golden_io import read_records
from oracle import literal
from test_oracle_scores import LN2
from test_oracle_select import unpack


def hier_problem(rng, H, C1, fan_lo, fan_hi, d, zero_frac=0.05):
    fans = rng.integers(fan_lo, fan_hi + 1, size=(H, C1))
    C2 = int(fans.sum(axis=1).max())
    # equal C2 per head: give the last coarse cluster the remainder
    fans[:, -1] += C2 - fans.sum(axis=1)
    co = np.zeros((H, C1 + 1), np.int32); co[:, 1:] = np.cumsum(fans, axis=1)
    cent2 = (rng.standard_normal((H, C2, d)) * 0.8).astype(np.float16)
    sizes2 = rng.integers(1, 7, size=(H, C2)).astype(np.int32)
    sizes2[rng.random((H, C2)) < zero_frac] = 0
    off2 = np.zeros((H, C2 + 1), np.int32); off2[:, 1:] = np.cumsum(sizes2, axis=1)
    cent1 = np.zeros((H, C1, d), np.float16); sizes1 = np.zeros((H, C1), np.int32)
    for h in range(H):
        for j in range(C1):
            sl = slice(co[h, j], co[h, j + 1])
            cent1[h, j] = cent2[h, sl].astype(np.float64).mean(0) if co[h, j + 1] > co[h, j] else 0
            sizes1[h, j] = sizes2[h, sl].sum()
    q = rng.standard_normal((1, H, d)).astype(np.float16)
    return q, cent1, sizes1, co, cent2, sizes2, off2


def test_hand_example_two_levels(oracle):
    g = read_records("eq1_hand_example.txt")["two_level"]
    d = 4
    q = np.zeros((1, 1, d), np.float16); q[..., 0] = 1
    c1 = np.zeros((1, 2, d), np.float16); c1[0, :, 0] = g["a1"]
    c2 = np.zeros((1, 4, d), np.float16); c2[0, :, 0] = g["a2"]; c2[0, :, 1] = [5, -7, 3, 1]
    N1 = np.asarray(g["N1"], np.int32)[None]; N2 = np.asarray(g["N2"], np.int32)[None]
    co = np.array([[0, 2, 4]], np.int32)
    off2 = np.concatenate([[0], np.cumsum(N2[0])]).astype(np.int32)[None]
    for T2key, keptkey in [("T2", "kept_fine"), ("T2_strict", "kept_fine_strict")]:
        r = oracle.hier_select(q, c1, N1, co, np.float32(g["T1"]), c2, N2, off2, np.float32(g[T2key]), LN2,
                               want_logits2=True)
        assert list(np.flatnonzero(unpack(r["mask1"], 2)[0, 0])) == [0]
        kept = [int(c) for c in g[keptkey]]
        assert list(np.flatnonzero(unpack(r["mask2"], 4)[0, 0])) == kept
        assert r["n_keys"][0, 0] == sum(N2[0, c] for c in kept)
        m1, D1, m2, D2 = r["stats"][0, 0].astype(np.float64)
        x2 = r["logits2"][0, 0].astype(np.float64)
        np.testing.assert_allclose(np.exp(x2[:2] - m2) / D2, g["S2"], rtol=2e-6)
        assert np.isnan(x2[2:]).all()
        np.testing.assert_allclose(np.exp(np.array(g["a1"]) * LN2 - m1) / D1, g["S1"], rtol=2e-6)
        k1, k2, S1, S2 = literal.hier_select(q[0, 0], c1[0], N1[0], co[0], np.float32(g["T1"][0]), c2[0], N2[0],
                                             np.float32(g[T2key][0]), LN2)
        np.testing.assert_allclose(S1, g["S1"], rtol=2e-6); np.testing.assert_allclose(S2[:2], g["S2"], rtol=2e-6)
        assert list(np.flatnonzero(k2)) == kept


@pytest.mark.parametrize("seed", range(4))
def test_keep_all_coarse_equals_one_level(oracle, seed):
    rng = np.random.default_rng(200 + seed)
    H, C1 = 2, 6
    q, c1, N1, co, c2, N2, off2 = hier_problem(rng, H, C1, 1, 5, 32)
    T2 = np.full(H, 0.02, np.float32)
    r = oracle.hier_select(q, c1, N1, co, np.full(H, -1.0, np.float32), c2, N2, off2, T2, 0.3)
    x, m, D = oracle.centroid_score(q[:, :, None], c2, N2, 0.3)
    mask, ranges, nr, nk = oracle.select(x, m, D, T2, N2, off2)
    # coarse clusters whose children are all empty have N1 = 0 and are dropped; their children are empty anyway
    np.testing.assert_array_equal(r["mask2"], mask[:, :, 0])
    np.testing.assert_array_equal(r["n_keys"], nk[:, :, 0])
    np.testing.assert_array_equal(r["ranges"], ranges[:, :, 0])


@pytest.mark.parametrize("seed", range(4))
def test_structure_and_bruteforce(oracle, seed):
    rng = np.random.default_rng(300 + seed)
    H, C1 = 3, 9
    q, c1, N1, co, c2, N2, off2 = hier_problem(rng, H, C1, 0, 6, 64)
    C2 = c2.shape[1]
    T1 = np.full(H, 0.012, np.float32); T2 = np.full(H, 0.03, np.float32)
    r = oracle.hier_select(q, c1, N1, co, T1, c2, N2, off2, T2, 0.3, want_logits2=True)
    k1 = unpack(r["mask1"], C1)[0]; k2 = unpack(r["mask2"], C2)[0]
    for h in range(H):
        cand = np.zeros(C2, bool)
        for j in np.flatnonzero(k1[h]):
            cand[co[h, j]:co[h, j + 1]] = True
        assert not (k2[h] & ~cand).any()                       # kept fine clusters are children of kept coarse ones
        x2 = r["logits2"][0, h].astype(np.float64)
        assert (np.isnan(x2) == ~cand).all()
        m2, D2 = r["stats"][0, h, 2:].astype(np.float64)
        if cand.any() and N2[h][cand].sum() > 0:
            S2 = np.exp(x2[cand] - m2) / D2
            assert (S2 * N2[h][cand]).sum() == pytest.approx(1.0, rel=1e-5)   # Eq. 3 normalised over candidates only
        l1, l2, S1, S2l = literal.hier_select(q[0, h], c1[h], N1[h], co[h], T1[h], c2[h], N2[h], T2[h], 0.3)
        near1 = literal.near_threshold(S1, T1[h])
        assert not ((k1[h] != l1) & ~near1).any()
        if (k1[h] == l1).all():
            near2 = literal.near_threshold(np.nan_to_num(S2l, nan=1.0), T2[h])
            assert not ((k2[h] != l2) & ~near2).any()
        assert r["n_keys"][0, h] == N2[h][k2[h]].sum() and r["n_ranges"][0, h] == k2[h].sum()
