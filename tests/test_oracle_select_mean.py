"""Pins for the oracle's prefill selection on averaged scores (Appendix D, "Prefill Stage")."""
import math

import numpy as np

from conftest import random_problem
from oracle import literal
from test_oracle_select import unpack


def offsets_of(sizes):
    off = np.zeros((sizes.shape[0], sizes.shape[1] + 1), np.int32)
    off[:, 1:] = np.cumsum(sizes, axis=1)
    return off


def run(oracle, logits, sizes, T, want_scores=False):
    """Statistics from the logits as Eq. 1 defines them (library calls, fp64 -> fp32), then the oracle."""
    logits = np.asarray(logits, np.float32)
    m = logits.max(axis=-1)
    D = (np.exp(logits.astype(np.float64) - m[..., None]) * sizes[None, :, None, :]).sum(-1).astype(np.float32)
    H = sizes.shape[0]
    thr = np.full(H, T, np.float32)
    return oracle.select_mean(logits, m, D, thr, sizes, offsets_of(sizes), want_scores=want_scores)


def test_two_token_closed_form(oracle):
    # Two clusters of one key each.  Token 1: logits (0, 0) -> S = (1/2, 1/2).  Token 2: logits (ln 3, 0)
    # -> S = (3/4, 1/4).  Averages: (5/8, 3/8).
    logits = np.array([[[[0.0, 0.0], [math.log(3.0), 0.0]]]], np.float32)       # [B=1, H=1, Lq=2, C=2]
    sizes = np.ones((1, 2), np.int32)
    mask, ranges, nr, nk, sbar = run(oracle, logits, sizes, 0.4, want_scores=True)
    np.testing.assert_allclose(sbar[0, 0], [0.625, 0.375], rtol=1e-6)
    assert unpack(mask, 2)[0, 0].tolist() == [True, False]
    assert nr[0, 0] == 1 and nk[0, 0] == 1 and ranges[0, 0, 0].tolist() == [0, 1]
    mask, _, nr, _ = run(oracle, logits, sizes, 0.3)
    assert unpack(mask, 2)[0, 0].tolist() == [True, True] and nr[0, 0] == 2
    mask, _, nr, _ = run(oracle, logits, sizes, 0.7)
    assert not mask.any() and nr[0, 0] == 0


def test_tie_is_dropped_and_sizes_weight_the_normaliser(oracle):
    # Equal logits, sizes (3, 1): S_i = 1/4 for both clusters and every token; 1/4 > 1/4 is false (strict '>').
    logits = np.zeros((1, 1, 5, 2), np.float32)
    sizes = np.array([[3, 1]], np.int32)
    mask, _, nr, nk, sbar = run(oracle, logits, sizes, 0.25, want_scores=True)
    np.testing.assert_array_equal(sbar[0, 0], [0.25, 0.25])
    assert nr[0, 0] == 0 and nk[0, 0] == 0 and not mask.any()
    mask, ranges, nr, nk = run(oracle, logits, sizes, np.nextafter(np.float32(0.25), np.float32(0)))
    assert nr[0, 0] == 2 and nk[0, 0] == 4 and ranges[0, 0, :2].tolist() == [[0, 3], [3, 1]]


def test_single_token_equals_per_query_rule(oracle):
    # Lq = 1: the average is the score itself, so the kept set is that of the per-query rule, except for
    # clusters next to the threshold (e_i > T*D and e_i/D > T round differently).
    rng = np.random.default_rng(5)
    H, C, d = 3, 90, 32
    cent, sizes, offsets, q = random_problem(rng, H, C, d, 1, zero_frac=0.1)
    x, m, D = oracle.centroid_score(q, cent, sizes, 0.4)
    for T in [1e-4, 3e-3, 2e-2]:
        thr = np.full(H, T, np.float32)
        mask1 = oracle.select(x, m, D, thr, sizes, offsets)[0][:, :, 0]
        mask2, ranges2, nr2, nk2 = oracle.select_mean(x, m, D, thr, sizes, offsets)
        k1, k2 = unpack(mask1, C), unpack(mask2, C)
        for b, h, c in np.argwhere(k1 != k2):
            S = literal.scores(q[b, h], cent[h], sizes[h], 0.4)[0]
            assert literal.near_threshold(S[c], T)
        np.testing.assert_array_equal(nk2, (k2 * sizes[None]).sum(-1))
        np.testing.assert_array_equal(nr2, k2.sum(-1))


def test_brute_force_literal_equations_and_invariants(oracle):
    rng = np.random.default_rng(6)
    H, C, d, Lq = 2, 45, 16, 7
    cent, sizes, offsets, q = random_problem(rng, H, C, d, Lq, zero_frac=0.15)
    x, m, D = oracle.centroid_score(q, cent, sizes, 0.5)
    for T in [0.0, 2e-3, 1e-2, 4e-2]:
        thr = np.full(H, T, np.float32)
        mask, ranges, nr, nk, sbar = oracle.select_mean(x, m, D, thr, sizes, offsets, want_scores=True)
        keep = unpack(mask, C)
        for h in range(H):
            ref_keep, ref_S = literal.select_mean(q[0, h], cent[h], sizes[h], T, 0.5)
            live = sizes[h] > 0
            np.testing.assert_allclose(sbar[0, h][live], ref_S[live], rtol=2e-6)
            for c in np.flatnonzero(keep[0, h] != ref_keep):
                assert literal.near_threshold(ref_S[c], T)
            # the averaged scores still sum to one when weighted by the cluster sizes
            assert abs((sbar[0, h] * sizes[h]).sum() - 1.0) < 1e-5
            ids = np.flatnonzero(keep[0, h])
            np.testing.assert_array_equal(ranges[0, h, :len(ids)], np.stack([offsets[h, ids], sizes[h, ids]], 1))
            assert nr[0, h] == len(ids) and nk[0, h] == sizes[h, ids].sum()
            assert not keep[0, h][~live].any()


def test_order_of_the_tokens_does_not_matter_and_copies_change_nothing(oracle):
    rng = np.random.default_rng(7)
    H, C, d, Lq = 2, 33, 16, 6
    cent, sizes, offsets, q = random_problem(rng, H, C, d, Lq)
    thr = np.full(H, 1.2e-2, np.float32)
    x, m, D = oracle.centroid_score(q, cent, sizes, 0.5)
    base = oracle.select_mean(x, m, D, thr, sizes, offsets, want_scores=True)
    perm = rng.permutation(Lq)
    x2, m2, D2 = oracle.centroid_score(q[:, :, perm], cent, sizes, 0.5)
    other = oracle.select_mean(x2, m2, D2, thr, sizes, offsets, want_scores=True)
    np.testing.assert_allclose(other[4], base[4], rtol=1e-12)
    np.testing.assert_array_equal(other[0], base[0])
    # every token twice: same averages, same set
    x3, m3, D3 = oracle.centroid_score(np.concatenate([q, q], axis=2), cent, sizes, 0.5)
    twice = oracle.select_mean(x3, m3, D3, thr, sizes, offsets, want_scores=True)
    np.testing.assert_allclose(twice[4], base[4], rtol=1e-12)
    np.testing.assert_array_equal(twice[0], base[0])
