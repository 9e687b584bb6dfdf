"""Pins for the oracle's attention over kept fixed keys + user keys (Sections 3.2 and 4.2)."""
import math

import numpy as np
import pytest
import torch

from oracle import literal

# scales that are exact fp32 values, so the fp64 references see the same number the oracle does
S02, S03, S07 = (float(np.float32(v)) for v in (0.2, 0.3, 0.7))


def make(rng, B, H, Lq, L, U, d):
    f = lambda *s: rng.standard_normal(s).astype(np.float16)
    return f(B, H, Lq, d), f(H, L, d), f(H, L, d), f(B, H, U, d), f(B, H, U, d)


def full_ranges(B, H, Lq, L, cap=4):
    r = np.zeros((B, H, Lq, cap, 2), np.int32)
    r[..., 0, 1] = L
    return r, np.ones((B, H, Lq), np.int32)


def test_keep_all_equals_dense_attention(oracle):
    rng = np.random.default_rng(21)
    B, H, Lq, L, U, d = 2, 3, 1, 77, 19, 128
    q, Kf, Vf, Ku, Vu = make(rng, B, H, Lq, L, U, d)
    sm = float(np.float32(1 / math.sqrt(d)))
    rg, nr = full_ranges(B, H, Lq, L)
    out, lse = oracle.sparse_attn(q, Kf, Vf, rg, nr, Ku, Vu, sm)
    for b in range(B):
        for h in range(H):
            K = np.concatenate([Kf[h], Ku[b, h]]); V = np.concatenate([Vf[h], Vu[b, h]])
            ref, ref_lse = literal.dense_attention(q[b, h], K, V, sm)
            np.testing.assert_allclose(out[b, h], ref, rtol=1e-10, atol=1e-12)
            np.testing.assert_allclose(lse[b, h], ref_lse, rtol=1e-12)
            t = lambda a: torch.from_numpy(a.astype(np.float64))
            sdpa = torch.nn.functional.scaled_dot_product_attention(t(q[b, h])[None], t(K)[None], t(V)[None], scale=sm)
            np.testing.assert_allclose(out[b, h], sdpa[0].numpy(), rtol=1e-9, atol=1e-11)


def test_keep_all_prefill_causal_user_block(oracle):
    # Fixed context fully visible; user key j visible to query t iff j <= t (user input follows the context).
    rng = np.random.default_rng(22)
    B, H, Lq, L, d = 1, 2, 9, 40, 32
    U = Lq
    q, Kf, Vf, Ku, Vu = make(rng, B, H, Lq, L, U, d)
    rg, nr = full_ranges(B, H, Lq, L)
    out, lse = oracle.sparse_attn(q, Kf, Vf, rg, nr, Ku, Vu, S02, causal_user=True)
    for h in range(H):
        for t in range(Lq):
            K = np.concatenate([Kf[h], Ku[0, h, :t + 1]]); V = np.concatenate([Vf[h], Vu[0, h, :t + 1]])
            ref, ref_lse = literal.dense_attention(q[0, h, t:t + 1], K, V, S02)
            np.testing.assert_allclose(out[0, h, t], ref[0], rtol=1e-10, atol=1e-12)
    # with an empty fixed selection, row 0 sees exactly user key 0
    out0, _ = oracle.sparse_attn(q, Kf, Vf, rg, np.zeros_like(nr), Ku, Vu, S02, causal_user=True)
    np.testing.assert_allclose(out0[0, :, 0], Vu[0, :, 0].astype(np.float64), rtol=1e-12)


def test_single_selected_key_returns_its_value(oracle):
    rng = np.random.default_rng(23)
    q, Kf, Vf, Ku, Vu = make(rng, 1, 2, 1, 30, 0, 16)
    rg = np.zeros((1, 2, 1, 3, 2), np.int32)
    rg[0, 0, 0, 0] = (17, 1); rg[0, 1, 0, 0] = (4, 1)
    out, lse = oracle.sparse_attn(q, Kf, Vf, rg, np.ones((1, 2, 1), np.int32), Ku, Vu, S07)
    np.testing.assert_allclose(out[0, 0, 0], Vf[0, 17].astype(np.float64), rtol=1e-12)
    np.testing.assert_allclose(out[0, 1, 0], Vf[1, 4].astype(np.float64), rtol=1e-12)
    s = S07 * float(q[0, 0, 0].astype(np.float64) @ Kf[0, 17].astype(np.float64))
    assert lse[0, 0, 0] == pytest.approx(s, rel=1e-12)


def test_nothing_visible_gives_zero_and_minus_inf(oracle):
    rng = np.random.default_rng(24)
    q, Kf, Vf, Ku, Vu = make(rng, 1, 1, 1, 10, 0, 8)
    out, lse = oracle.sparse_attn(q, Kf, Vf, np.zeros((1, 1, 1, 2, 2), np.int32), np.zeros((1, 1, 1), np.int32),
                                  Ku, Vu, 1.0)
    assert (out == 0).all() and np.isneginf(lse).all()


def test_constant_values_and_permutation(oracle):
    # softmax weights sum to 1: constant V gives that constant; key order does not matter.
    rng = np.random.default_rng(25)
    B, H, Lq, L, U, d = 1, 1, 2, 50, 6, 16
    q, Kf, Vf, Ku, Vu = make(rng, B, H, Lq, L, U, d)
    rg = np.zeros((1, 1, Lq, 4, 2), np.int32)
    rg[..., 0, :] = (3, 10); rg[..., 1, :] = (20, 7); rg[..., 2, :] = (40, 10)
    nr = np.full((1, 1, Lq), 3, np.int32)
    out, lse = oracle.sparse_attn(q, Kf, np.full_like(Vf, 2.5), rg, nr, Ku, np.full_like(Vu, 2.5), S03)
    np.testing.assert_allclose(out, 2.5, rtol=1e-12)
    out, lse = oracle.sparse_attn(q, Kf, Vf, rg, nr, Ku, Vu, S03)
    idx = np.concatenate([np.arange(3, 13), np.arange(20, 27), np.arange(40, 50)])
    perm = rng.permutation(len(idx))
    K = np.concatenate([Kf[0, idx][perm], Ku[0, 0]]); V = np.concatenate([Vf[0, idx][perm], Vu[0, 0]])
    ref, ref_lse = literal.dense_attention(q[0, 0], K, V, S03)
    np.testing.assert_allclose(out[0, 0], ref, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(lse[0, 0], ref_lse, rtol=1e-12)


def test_split_and_merge_invariant(oracle):
    # Section 4.2 (two-phase split-KV): partial results over any partition of the key set, merged with
    # weights exp(lse_c - lse*), equal the unsplit result.
    rng = np.random.default_rng(26)
    q, Kf, Vf, Ku, Vu = make(rng, 1, 2, 1, 64, 5, 32)
    def run(ranges, with_user):
        rg = np.zeros((1, 2, 1, 4, 2), np.int32)
        for i, r in enumerate(ranges):
            rg[:, :, :, i] = r
        ku, vu = (Ku, Vu) if with_user else (Ku[:, :, :0], Vu[:, :, :0])
        return oracle.sparse_attn(q, Kf, Vf, rg, np.full((1, 2, 1), len(ranges), np.int32), ku, vu, 0.25)
    whole, lse = run([(0, 20), (30, 11), (50, 14)], True)
    parts = [run([(0, 20)], False), run([(30, 11), (50, 14)], False), run([], True)]
    L = np.stack([p[1] for p in parts]); O = np.stack([p[0] for p in parts])
    Lmax = L.max(0)
    wgt = np.exp(L - Lmax)
    merged = (wgt[..., None] * O).sum(0) / wgt.sum(0)[..., None]
    np.testing.assert_allclose(merged, whole, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(Lmax + np.log(wgt.sum(0)), lse, rtol=1e-12)


def test_row_sampling_matches_full(oracle):
    rng = np.random.default_rng(27)
    B, H, Lq, L, U, d = 1, 2, 6, 30, 6, 16
    q, Kf, Vf, Ku, Vu = make(rng, B, H, Lq, L, U, d)
    rg, nr = full_ranges(B, H, Lq, L)
    full, _ = oracle.sparse_attn(q, Kf, Vf, rg, nr, Ku, Vu, S02, causal_user=True)
    sel = np.zeros((B, H, Lq), bool); sel[0, 1, 4] = True
    part, _ = oracle.sparse_attn(q, Kf, Vf, rg, nr, Ku, Vu, S02, causal_user=True, row_sel=sel)
    np.testing.assert_array_equal(part[0, 1, 4], full[0, 1, 4])
    assert np.isnan(part[0, 0, 0]).all()
