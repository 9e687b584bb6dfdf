"""Pins of the offline clustering oracle (Section 3.1: K-means on normalised key vectors, cluster mean as the
centroid): a hand-checkable example, brute force with literally written squared distances, Lloyd's monotone
objective, fixed points, and the layout's bookkeeping."""
import numpy as np
import pytest

from oracle import clustering as cl


def test_two_clusters_by_hand():
    # points on a line (d = 2, second coordinate 0): centres at 0 and 10
    X = np.array([[-1, 0], [0, 0], [1, 0], [4, 0], [6, 0], [9, 0], [11, 0]], np.float16)
    c = np.array([[0, 0], [10, 0]], np.float16)
    a, margin = cl.assign(X, c)
    assert a.tolist() == [0, 0, 0, 0, 1, 1, 1]                  # the boundary is at 5
    # score = x.c - c^2/2: for x = 4 the scores are 0 and 40 - 50 = -10
    assert margin[3] == pytest.approx(10.0)
    new, counts = cl.update(X, a, c)
    assert counts.tolist() == [4, 3]
    np.testing.assert_allclose(new.astype(np.float64), [[1.0, 0], [26 / 3, 0]], rtol=1e-3)
    # a tie (x = 5) goes to the lower index
    a2, m2 = cl.assign(np.array([[5, 0]], np.float16), c)
    assert a2.tolist() == [0] and m2[0] == 0.0
    # a centre without members keeps its value
    new2, cnt2 = cl.update(X[:3], np.zeros(3, np.int32), c)
    assert cnt2.tolist() == [3, 0] and new2[1].tolist() == [10, 0]


@pytest.mark.parametrize("seed", range(3))
def test_assignment_is_the_literal_nearest_centre(seed):
    rng = np.random.default_rng(900 + seed)
    X = cl.normalize_rows(rng.standard_normal((300, 16)).astype(np.float16))
    c = (rng.standard_normal((11, 16)) * 0.4).astype(np.float16)
    a, margin = cl.assign(X, c)
    d2 = ((X.astype(np.float64)[:, None, :] - c.astype(np.float64)[None, :, :]) ** 2).sum(-1)   # |x - c|^2 written out
    lit = d2.argmin(axis=1)
    clear = margin > 1e-9
    np.testing.assert_array_equal(a[clear], lit[clear])
    assert clear.mean() > 0.99
    # unit rows
    np.testing.assert_allclose((X.astype(np.float64) ** 2).sum(-1), 1.0, atol=2e-3)


def test_lloyd_objective_never_increases_and_reaches_a_fixed_point():
    rng = np.random.default_rng(910)
    centres = rng.standard_normal((8, 32))
    X = cl.normalize_rows((centres[rng.integers(0, 8, 2000)] + 0.3 * rng.standard_normal((2000, 32))).astype(np.float16))
    c = X[rng.choice(2000, 8, replace=False)].copy()
    objs = []
    for _ in range(30):
        a, c_new, n, obj = cl.lloyd_step(X, c)
        objs.append(obj)
        if np.array_equal(c_new, c):
            break
        c = c_new
    # (centres are rounded to fp16 after every update, so allow that rounding in the comparison)
    assert all(b <= a * (1 + 1e-3) for a, b in zip(objs, objs[1:])), objs
    assert objs[-1] < 0.7 * objs[0]
    a2, c2, n2, _ = cl.lloyd_step(X, c)                         # at the fixed point nothing moves
    np.testing.assert_array_equal(c2, c)
    assert n2.sum() == 2000


def test_layout_groups_keys_by_cluster_and_averages_raw_keys():
    rng = np.random.default_rng(920)
    K = (rng.standard_normal((500, 8)) * 3).astype(np.float16)
    a = rng.integers(0, 13, 500).astype(np.int32)
    a[a == 7] = 6                                               # cluster 7 is empty
    perm, sizes, offsets, cent = cl.layout(K, a, 13)
    assert sorted(perm.tolist()) == list(range(500)) and sizes[7] == 0 and offsets[-1] == 500
    for c in range(13):
        seg = perm[offsets[c]:offsets[c + 1]]
        assert (a[seg] == c).all() and (np.diff(seg) > 0).all()  # grouped, ascending key index inside a cluster
        if len(seg):
            np.testing.assert_allclose(cent[c].astype(np.float64), K[seg].astype(np.float64).mean(0), atol=4e-3)
    assert (cent[7] == 0).all()


def test_nesting_keeps_every_key_under_the_coarse_cluster_of_its_fine_cluster():
    rng = np.random.default_rng(930)
    L, C2, C1 = 3000, 60, 7
    a_fine = rng.integers(0, C2, L).astype(np.int32)
    a_coarse = rng.integers(0, C1, C2).astype(np.int32)          # coarse cluster of each fine cluster
    a_coarse[a_coarse == 4] = 3                                  # coarse cluster 4 has no children
    perm_c, fan, co, _ = cl.layout(np.zeros((C2, 2), np.float16), a_coarse, C1)
    a_new, sizes, offsets, perm, sizes_c = cl.nest(a_fine, perm_c, co, C2)
    parent_new = np.searchsorted(co, a_new, side="right") - 1    # coarse cluster whose child range holds the new id
    np.testing.assert_array_equal(parent_new, a_coarse[a_fine])
    np.testing.assert_array_equal(sizes_c, np.bincount(a_coarse[a_fine], minlength=C1))
    assert sizes_c[4] == 0 and sizes_c.sum() == L
    np.testing.assert_array_equal(sizes[a_new[:50]], np.bincount(a_fine, minlength=C2)[a_fine[:50]])   # same clusters, renamed
    for c in range(C2):
        seg = perm[offsets[c]:offsets[c + 1]]
        assert (a_new[seg] == c).all() and (np.diff(seg) > 0).all()


def test_nesting_by_hand():
    # 4 fine clusters; coarse 0 = {fine 2, fine 0}, coarse 1 = {fine 3, fine 1} (perm_coarse order)
    a_new, sizes, offsets, perm, sizes_c = cl.nest(np.array([0, 1, 2, 3, 3, 0]), np.array([2, 0, 3, 1]),
                                                   np.array([0, 2, 4]), 4)
    assert a_new.tolist() == [1, 3, 0, 2, 2, 1]
    assert sizes.tolist() == [1, 2, 2, 1] and offsets.tolist() == [0, 1, 3, 5, 6]
    assert perm.tolist() == [2, 0, 5, 3, 4, 1] and sizes_c.tolist() == [3, 3]
