"""GPU parity of the lookup through any number of centroid levels (sq_multilevel_select, sq_multilevel_decode_step)
against the oracle: every level's kept set bit-exact outside the near-threshold band (a band disagreement at one
level excuses the levels below it, which then see other candidates), counts, ranges, attention."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import ATTN_ATOL, dev, unpack_mask
from oracle import literal
from test_oracle_multilevel import three_level_problem, with_thresholds

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sq():
    from paper_2411_09688_amd import binding
    binding.lib()
    return binding


def calibrate(q, levels, sm_scale, fracs):
    """Per-head thresholds that keep about fracs[k] of level k's candidates (quantiles of the literal fp64 scores,
    level after level; a negative fraction means keep everything)."""
    H = q.shape[1]
    levels = [dict(l, thresh=np.full(H, -1.0, np.float32)) for l in levels]
    for k, f in enumerate(fracs):
        if f < 0:
            continue
        for h in range(H):
            lit = literal.multilevel_select(q[0, h], [(l["centroids"][h], l["sizes"][h], l["child_offsets"][h],
                                                       l["thresh"][h]) for l in levels], sm_scale)
            S = lit[k][1]
            S = np.sort(S[~np.isnan(S) & (levels[k]["sizes"][h] > 0)])
            i = min(len(S) - 2, max(0, int(round(len(S) * (1 - f))) - 1))
            levels[k]["thresh"][h] = np.float32(np.sqrt(S[i] * S[i + 1]))      # between two scores
    return levels


def gpu_levels(levels):
    return [(dev(l["centroids"]), dev(l["sizes"]), dev(l["child_offsets"]), dev(l["thresh"])) for l in levels]


def run_select(sq, q, levels, sm_scale, L):
    B, H, d = q.shape
    Cl = levels[-1]["centroids"].shape[1]
    sh = sq.make_shape(B, H, L, Cl, 1, 0, sm_scale)
    D = "cuda:0"
    masks = [torch.zeros(B, H, (l["centroids"].shape[1] + 31) // 32, dtype=torch.int32, device=D) for l in levels]
    ranges = torch.zeros(B, H, 1, Cl, 2, dtype=torch.int32, device=D)
    nr = torch.zeros(B, H, 1, dtype=torch.int32, device=D)
    nk = torch.zeros(B, H, 1, dtype=torch.int32, device=D)
    ws = sq.workspace(sh, sq.SQ_CALL_MULTILEVEL_SELECT, torch.device(D))
    sq.sq_multilevel_select(sh, gpu_levels(levels), dev(q.reshape(B, H, 1, d)), masks, ranges, nr, nk, ws)
    torch.cuda.synchronize()
    return ([m.cpu().numpy() for m in masks], ranges.cpu().numpy()[:, :, 0], nr.cpu().numpy()[:, :, 0],
            nk.cpu().numpy()[:, :, 0])


def check_against_oracle(q, levels, sm_scale, got, label):
    """Returns the (b, h) rows whose kept sets agree with the oracle at every level."""
    masks, ranges, nr, nk = got
    ref = oracle.multilevel_select(q, levels, sm_scale)
    B, H, _ = q.shape
    same = []
    for b in range(B):
        for h in range(H):
            lit = literal.multilevel_select(q[b, h], [(l["centroids"][h], l["sizes"][h], l["child_offsets"][h],
                                                       l["thresh"][h]) for l in levels], sm_scale)
            agree = True
            for k, l in enumerate(levels):
                Ck = l["centroids"].shape[1]
                g = unpack_mask(masks[k], Ck)[b, h]
                o = unpack_mask(ref["masks"][k], Ck)[b, h]
                if agree:
                    dif = np.flatnonzero(g != o)
                    S = np.nan_to_num(lit[k][1], nan=1.0)
                    assert literal.near_threshold(S[dif], l["thresh"][h]).all(), (label, b, h, "level", k, dif)
                    if len(dif):
                        print(f"[near-threshold clusters {label}] b{b} h{h} level {k}: {dif.tolist()}")
                        agree = False
                if k > 0:                                         # kept clusters are children of kept parents
                    par = unpack_mask(masks[k - 1], levels[k - 1]["centroids"].shape[1])[b, h]
                    cand = np.zeros(Ck, bool)
                    co = levels[k - 1]["child_offsets"][h]
                    for j in np.flatnonzero(par):
                        cand[co[j]:co[j + 1]] = True
                    assert not (g & ~cand).any(), (label, b, h, k)
            last = levels[-1]
            ids = np.flatnonzero(unpack_mask(masks[-1], last["centroids"].shape[1])[b, h])
            assert nr[b, h] == len(ids) and nk[b, h] == last["sizes"][h][ids].sum()
            np.testing.assert_array_equal(ranges[b, h, :len(ids)],
                                          np.stack([last["child_offsets"][h][ids], last["sizes"][h][ids]], 1))
            if agree:
                same.append((b, h))
    return same


@pytest.mark.parametrize("seed,H,C0,fan01,fan12,fracs", [
    (0, 2, 4, 3, (1, 5), (0.5, 0.5, 0.5)),
    (1, 3, 6, 8, (0, 9), (0.5, 0.4, 0.3)),
    (2, 1, 20, 10, (10, 30), (0.7, 0.6, 0.5)),              # over a thousand kept candidates: several selection steps
    (3, 2, 8, 16, (8, 8), (-1, 0.3, 0.4)),                  # the top level keeps everything
    (4, 1, 30, 60, (1, 3), (0.9, 0.8, 0.5)),                # over a thousand candidates at the MIDDLE level too
])
def test_three_level_select(sq, seed, H, C0, fan01, fan12, fracs):
    rng = np.random.default_rng(700 + seed)
    q, levels = three_level_problem(rng, H, C0, fan01, fan12, 128)
    levels = calibrate(q, levels, 0.3, fracs)
    L = int(levels[-1]["sizes"].sum(axis=1).max())
    got = run_select(sq, q[0][None], levels, 0.3, L)
    same = check_against_oracle(q[0][None], levels, 0.3, got, f"3-level seed {seed}")
    assert len(same) >= 1 and got[3].sum() > 0


def test_two_and_one_level_match_the_dedicated_calls(sq):
    rng = np.random.default_rng(710)
    H = 2
    q, levels = three_level_problem(rng, H, 5, 4, (2, 9), 128)
    levels = calibrate(q, levels, 0.3, (0.5, 0.5, 0.4))
    L = int(levels[-1]["sizes"].sum(axis=1).max())
    for sub in (calibrate(q, levels[1:], 0.3, (0.5, 0.4)), calibrate(q, levels[2:], 0.3, (0.3,))):
        got = run_select(sq, q[0][None], sub, 0.3, L)
        check_against_oracle(q[0][None], sub, 0.3, got, f"{len(sub)}-level")
    # two levels through sq_hier_select: bit-identical outputs
    from test_gpu_hier import run_hier_select
    l1, l2 = calibrate(q, levels[1:], 0.3, (0.5, 0.4))
    got = run_select(sq, q[0][None], [l1, l2], 0.3, L)
    sh, t = run_hier_select(sq, 1, H, l1["centroids"].shape[1], l2["centroids"].shape[1], L, q[0][None], l1["centroids"],
                            l1["sizes"], l1["child_offsets"], l1["thresh"], l2["centroids"], l2["sizes"],
                            l2["child_offsets"], l2["thresh"], 0.3)
    np.testing.assert_array_equal(got[0][0], t["m1"].cpu().numpy())
    np.testing.assert_array_equal(got[0][1], t["m2"].cpu().numpy())
    np.testing.assert_array_equal(got[3], t["nk"].cpu().numpy()[:, :, 0])


def test_three_level_decode_step(sq):
    rng = np.random.default_rng(720)
    H, U, d = 2, 37, 128
    q, levels = three_level_problem(rng, H, 6, 6, (3, 12), d)
    levels = calibrate(q, levels, 0.3, (0.5, 0.5, 0.5))
    L = int(levels[-1]["sizes"].sum(axis=1).max())
    # keys and values: every head gets L rows (heads with fewer keys leave the tail unused)
    Kf = rng.standard_normal((H, L, d)).astype(np.float16); Vf = rng.standard_normal((H, L, d)).astype(np.float16)
    Ku = rng.standard_normal((1, H, U, d)).astype(np.float16); Vu = rng.standard_normal((1, H, U, d)).astype(np.float16)
    Cl = levels[-1]["centroids"].shape[1]
    sh = sq.make_shape(1, H, L, Cl, 1, U, 0.3)
    D = "cuda:0"
    out = torch.full((1, H, 1, d), 7.0, dtype=torch.float16, device=D)
    lse = torch.zeros(1, H, 1, dtype=torch.float32, device=D)
    mask = torch.zeros(1, H, (Cl + 31) // 32, dtype=torch.int32, device=D)
    nk = torch.zeros(1, H, 1, dtype=torch.int32, device=D)
    ws = sq.workspace(sh, sq.SQ_CALL_MULTILEVEL_DECODE_STEP, torch.device(D))
    sq.sq_multilevel_decode_step(sh, gpu_levels(levels), dev(q[0][None].reshape(1, H, 1, d)), dev(Kf), dev(Vf), dev(Ku),
                                 dev(Vu), out, lse, mask, nk, ws)
    torch.cuda.synchronize()
    got_sel = run_select(sq, q[0][None], levels, 0.3, L)
    np.testing.assert_array_equal(mask.cpu().numpy(), got_sel[0][-1])      # the step selects what the lookup selects
    np.testing.assert_array_equal(nk.cpu().numpy()[:, :, 0], got_sel[3])
    check_against_oracle(q[0][None], levels, 0.3, got_sel, "3-level step")
    # attention over the GPU's selection, by the oracle
    keep = unpack_mask(mask.cpu().numpy(), Cl)
    last = levels[-1]
    ranges = np.zeros((1, H, 1, Cl, 2), np.int32); n_r = np.zeros((1, H, 1), np.int32)
    for h in range(H):
        ids = np.flatnonzero(keep[0, h])
        ranges[0, h, 0, :len(ids), 0] = last["child_offsets"][h][ids]
        ranges[0, h, 0, :len(ids), 1] = last["sizes"][h][ids]
        n_r[0, h, 0] = len(ids)
    ro, rl = oracle.sparse_attn(q[0][None].reshape(1, H, 1, d), Kf, Vf, ranges, n_r, Ku, Vu, 0.3)
    err = np.abs(out.cpu().numpy().astype(np.float64) - ro).max()
    assert err <= ATTN_ATOL, err
    np.testing.assert_allclose(lse.cpu().numpy(), rl, atol=1e-4, rtol=1e-5)
    assert nk.cpu().numpy().sum() > 0


def test_level_arguments_are_validated(sq):
    rng = np.random.default_rng(730)
    q, levels = three_level_problem(rng, 1, 3, 2, (1, 3), 128)
    levels = with_thresholds(levels, (0.1, 0.1, 0.1))
    L = int(levels[-1]["sizes"].sum(axis=1).max())
    with pytest.raises(sq.SqError) as e:                                   # more levels than supported
        run_select(sq, q[0][None], levels + levels, 0.3, L)
    assert e.value.code == sq.SQ_ERR_INVALID_ARG
    # a level with more clusters than the last one (= shape->C) is rejected
    big = dict(levels[0])
    Cl = levels[-1]["centroids"].shape[1]
    big["centroids"] = np.zeros((1, Cl + 1, 128), np.float16)
    big["sizes"] = np.ones((1, Cl + 1), np.int32)
    big["child_offsets"] = np.zeros((1, Cl + 2), np.int32)
    with pytest.raises(sq.SqError) as e:
        run_select(sq, q[0][None], [big, levels[-1]], 0.3, L)
    assert e.value.code == sq.SQ_ERR_INVALID_ARG
