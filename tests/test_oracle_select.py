"""Pins for the oracle's threshold rule and key ranges (Sections 3.2, 4.1, 4.2; Appendix D)."""
import numpy as np
import pytest

from conftest import random_problem
from golden_io import read_records
from oracle import literal
from test_oracle_scores import LN2, hand_problem


def run_select(oracle, q, cent, sizes, offsets, T, sm_scale):
    x, m, D = oracle.centroid_score(q, cent, sizes, sm_scale)
    H = cent.shape[0]
    thr = np.full(H, T, np.float32) if np.isscalar(T) else np.asarray(T, np.float32)
    return oracle.select(x, m, D, thr, sizes, offsets)


def unpack(mask, C):
    bits = (mask[..., :, None] >> np.arange(32, dtype=np.uint32)) & 1
    return bits.reshape(*mask.shape[:-1], -1)[..., :C].astype(bool)


def test_hand_example_selection(oracle):
    g = read_records("eq1_hand_example.txt")["one_level"]
    q, cent = hand_problem(g["a"])
    sizes = np.asarray(g["N"], np.int32)[None]
    offsets = np.concatenate([[0], np.cumsum(sizes[0])]).astype(np.int32)[None]
    mask, ranges, nr, nk = run_select(oracle, q, cent, sizes, offsets, g["T"][0], LN2)
    kept = [int(c) for c in g["kept"]]
    assert list(np.flatnonzero(unpack(mask, 4)[0, 0, 0])) == kept
    assert nr[0, 0, 0] == len(kept) and nk[0, 0, 0] == sum(sizes[0, c] for c in kept)
    assert ranges[0, 0, 0, :2].tolist() == [[offsets[0, c], sizes[0, c]] for c in kept]


def test_tie_is_dropped(oracle):
    # Equal centroids, L = 64 keys: e_i = 1, D = 64, T = 1/64 exactly -> 1 > 1 is false (strict '>').
    cent = np.ones((1, 8, 4), np.float16)
    sizes = np.full((1, 8), 8, np.int32)
    offsets = (np.arange(9, dtype=np.int32) * 8)[None]
    q = np.ones((1, 1, 1, 4), np.float16)
    mask, _, nr, nk = run_select(oracle, q, cent, sizes, offsets, 1.0 / 64, 1.0)
    assert nr[0, 0, 0] == 0 and nk[0, 0, 0] == 0 and not mask.any()
    mask, _, nr, nk = run_select(oracle, q, cent, sizes, offsets, np.nextafter(np.float32(1 / 64), 0), 1.0)
    assert nr[0, 0, 0] == 8 and nk[0, 0, 0] == 64


def test_monotone_nonempty_and_keep_all(oracle):
    rng = np.random.default_rng(11)
    H, C, d, nq = 3, 70, 32, 4
    cent, sizes, offsets, q = random_problem(rng, H, C, d, nq, zero_frac=0.1)
    L = sizes.sum(axis=1)
    prev = None
    for T in [-1.0, 0.0, 1e-4, 3e-3, 1e-2, 5e-2, 0.3, 2.0]:
        mask, ranges, nr, nk = run_select(oracle, q, cent, sizes, offsets, T, 0.4)
        keep = unpack(mask, C)
        if prev is not None:
            assert not (keep & ~prev).any()           # T_a < T_b  =>  sel(T_b) subset of sel(T_a)
        prev = keep
        assert not keep[:, :, :, :][..., :].transpose(0, 2, 1, 3)[..., sizes == 0].any()   # empty clusters never kept
        np.testing.assert_array_equal(nk, (keep * sizes[None, :, None, :]).sum(-1))
        np.testing.assert_array_equal(nr, keep.sum(-1))
        if T < 0:
            assert (keep == (sizes > 0)[None, :, None, :]).all()                 # negative T keeps everything
            np.testing.assert_array_equal(nk[0, :, 0], L)
    # T below 1/L always keeps something, because max_i S_i >= 1 / sum N.
    mask, *_ = run_select(oracle, q, cent, sizes, offsets, (0.999 / L).astype(np.float32), 0.4)
    assert unpack(mask, C).any(-1).all()
    # T above every score keeps nothing.
    assert prev.sum() == 0


def test_ranges_are_the_kept_clusters_key_intervals(oracle):
    rng = np.random.default_rng(12)
    H, C = 2, 45
    cent, sizes, offsets, q = random_problem(rng, H, C, 16, 3, max_size=9, zero_frac=0.15)
    mask, ranges, nr, nk = run_select(oracle, q, cent, sizes, offsets, 0.01, 0.5)
    keep = unpack(mask, C)
    for h in range(H):
        for t in range(3):
            n = nr[0, h, t]
            r = ranges[0, h, t, :n]
            ids = np.flatnonzero(keep[0, h, t])
            np.testing.assert_array_equal(r[:, 0], offsets[h, ids])
            np.testing.assert_array_equal(r[:, 1], sizes[h, ids])
            assert (r[:, 1] > 0).all() and (r[:, 0] >= 0).all() and (r[:, 0] + r[:, 1] <= offsets[h, -1]).all()
            assert (r[1:, 0] >= r[:-1, 0] + r[:-1, 1]).all()          # ascending and disjoint


@pytest.mark.parametrize("seed", range(6))
def test_bruteforce_against_literal_equation(oracle, seed):
    # Eq. 1 evaluated literally in fp64 and compared with T for every cluster of small random problems.
    rng = np.random.default_rng(100 + seed)
    H, C, d, nq = 2, int(rng.integers(3, 90)), int(rng.choice([8, 64, 128])), 5
    cent, sizes, offsets, q = random_problem(rng, H, C, d, nq, max_size=12, zero_frac=0.1)
    T = float(rng.choice([2e-3, 1e-2, 3e-2]))
    sm = float(rng.choice([0.1, 0.35]))
    mask, *_ = run_select(oracle, q, cent, sizes, offsets, T, sm)
    keep = unpack(mask, C)
    for h in range(H):
        ref, S = literal.select(q[0, h], cent[h], sizes[h], np.float32(T), sm)
        near = literal.near_threshold(S, np.float32(T))
        bad = (keep[0, h] != ref) & ~near
        assert not bad.any(), (h, np.argwhere(bad))
