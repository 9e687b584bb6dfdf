"""Pins for the oracle's cluster scores (Eq. 1, Section 3.2; max-subtracted form of Appendix D)."""
import math

import numpy as np
import pytest
import scipy.special

from conftest import random_problem
from golden_io import read_records
from oracle import literal

LN2 = float(np.float32(math.log(2.0)))


def S_from(oracle, q, cent, sizes, sm_scale):
    x, m, D = oracle.centroid_score(q, cent, sizes, sm_scale)
    return np.exp(x.astype(np.float64) - m[..., None]) / D[..., None].astype(np.float64), x, m, D


def hand_problem(a, d=4, seed=3):
    rng = np.random.default_rng(seed)
    cent = rng.integers(-3, 4, size=(1, len(a), d)).astype(np.float16)
    cent[0, :, 0] = np.asarray(a, dtype=np.float16)
    q = np.zeros((1, 1, 1, d), np.float16)
    q[..., 0] = 1.0
    return q, cent


def test_hand_example_eq1(oracle):
    g = read_records("eq1_hand_example.txt")["one_level"]
    q, cent = hand_problem(g["a"])
    sizes = np.asarray(g["N"], np.int32)[None]
    S, *_ = S_from(oracle, q, cent, sizes, LN2)
    np.testing.assert_allclose(S[0, 0, 0], g["S"], rtol=2e-6)
    np.testing.assert_allclose(literal.scores(q[0, 0], cent[0], sizes[0], LN2)[0], g["S"], rtol=2e-6)


@pytest.mark.parametrize("H,C,d,nq", [(2, 7, 16, 3), (3, 33, 128, 2), (1, 130, 64, 5)])
def test_size_weighted_scores_sum_to_one(oracle, H, C, d, nq):
    # Eq. 1: sum_i N_i S_i = 1 by construction of the denominator.
    rng = np.random.default_rng(C)
    cent, sizes, _, q = random_problem(rng, H, C, d, nq, zero_frac=0.1)
    S, *_ = S_from(oracle, q, cent, sizes, 0.3)
    np.testing.assert_allclose((S * sizes[None, :, None, :]).sum(-1), 1.0, rtol=1e-5)


def test_shift_invariance(oracle):
    # Adding one vector to every centroid multiplies numerator and denominator by the same factor.
    rng = np.random.default_rng(5)
    H, C, d = 2, 19, 32
    cent = rng.integers(-4, 5, size=(H, C, d)).astype(np.float16)
    shift = rng.integers(-3, 4, size=(H, 1, d)).astype(np.float16)
    sizes = rng.integers(1, 9, size=(H, C)).astype(np.int32)
    q = (rng.integers(-4, 5, size=(1, H, 2, d)) / 4).astype(np.float16)
    S0, x0, m0, _ = S_from(oracle, q, cent, sizes, 0.25)
    S1, x1, m1, _ = S_from(oracle, q, cent + shift, sizes, 0.25)
    assert not np.allclose(m0, m1)          # the shift really moved the logits
    np.testing.assert_allclose(S1, S0, rtol=1e-5)


def test_equal_centroids_give_one_over_L(oracle):
    rng = np.random.default_rng(6)
    H, C, d = 1, 12, 16
    row = rng.standard_normal(d).astype(np.float16)
    cent = np.broadcast_to(row, (H, C, d)).copy()
    sizes = rng.integers(1, 50, size=(H, C)).astype(np.int32)
    q = rng.standard_normal((1, H, 1, d)).astype(np.float16)
    S, *_ = S_from(oracle, q, cent, sizes, 1.0)
    np.testing.assert_allclose(S, 1.0 / sizes.sum(), rtol=1e-6)


def test_single_cluster(oracle):
    q = np.ones((1, 1, 1, 8), np.float16)
    cent = np.full((1, 1, 8), 0.5, np.float16)
    S, x, m, D = S_from(oracle, q, cent, np.array([[37]], np.int32), 0.5)
    assert x[0, 0, 0, 0] == pytest.approx(0.5 * 4.0) and m[0, 0, 0] == x[0, 0, 0, 0] and D[0, 0, 0] == 37.0
    np.testing.assert_allclose(S, 1.0 / 37.0, rtol=1e-7)


def test_one_key_per_cluster_is_library_softmax(oracle):
    # C = L, N_i = 1, C_i = k_i: S_i is the true attention probability (the "Ideal" lookup of Appendix H).
    rng = np.random.default_rng(7)
    L, d, nq = 57, 128, 4
    K = rng.standard_normal((1, L, d)).astype(np.float16)
    q = rng.standard_normal((1, 1, nq, d)).astype(np.float16)
    sm = float(np.float32(1 / math.sqrt(d)))
    S, *_ = S_from(oracle, q, K, np.ones((1, L), np.int32), sm)
    ref = scipy.special.softmax(sm * (q[0, 0].astype(np.float64) @ K[0].astype(np.float64).T), axis=1)
    np.testing.assert_allclose(S[0, 0], ref, rtol=2e-5)
    np.testing.assert_allclose(literal.scores(q[0, 0], K[0], np.ones(L), sm), ref, rtol=1e-12)


def test_logits_are_scaled_dot_products_not_transposed(oracle):
    # x[b,h,t,i] = sm_scale * q[b,h,t,:] . C[h,i,:]  with every index distinct.
    rng = np.random.default_rng(8)
    B, H, Lq, C, d = 2, 3, 4, 5, 8
    q = rng.integers(-3, 4, size=(B, H, Lq, d)).astype(np.float16)
    cent = rng.integers(-3, 4, size=(H, C, d)).astype(np.float16)
    x, m, D = oracle.centroid_score(q, cent, np.ones((H, C), np.int32), 0.5)
    ref = 0.5 * np.einsum("bhtd,hcd->bhtc", q.astype(np.float64), cent.astype(np.float64))
    np.testing.assert_array_equal(x, ref.astype(np.float32))     # small integers: exact in fp32
    np.testing.assert_array_equal(m, ref.max(-1).astype(np.float32))


def test_c_oracle_matches_literal_fp64(oracle):
    rng = np.random.default_rng(9)
    for (H, C, d, nq) in [(2, 40, 128, 6), (1, 9, 24, 3)]:
        cent, sizes, _, q = random_problem(rng, H, C, d, nq, max_size=40, zero_frac=0.05)
        S, *_ = S_from(oracle, q, cent, sizes, 0.2)
        for h in range(H):
            ref = literal.scores(q[0, h], cent[h], sizes[h], 0.2)
            np.testing.assert_allclose(S[0, h], ref, rtol=2e-5)


def test_zero_size_cluster_with_largest_logit_is_ignored(oracle):
    q = np.zeros((1, 1, 1, 4), np.float16); q[..., 0] = 1
    cent = np.zeros((1, 3, 4), np.float16); cent[0, :, 0] = [1, 60, 2]   # the empty cluster has a huge logit
    sizes = np.array([[2, 0, 3]], np.int32)
    S, x, m, D = S_from(oracle, q, cent, sizes, LN2)
    assert m[0, 0, 0] == pytest.approx(2 * LN2)
    np.testing.assert_allclose(S[0, 0, 0, [0, 2]], [2 / 16, 4 / 16], rtol=1e-6)   # D = 2*2 + 3*4
