"""The synthetic workload generator: layout invariants and calibration (host logic only)."""
import numpy as np
import pytest

from paper_2411_09688_amd import workload as wl


@pytest.fixture(scope="module")
def cfg1(oracle):
    return wl.calibrate(wl.make_config("cfg1_tiny_decode"), oracle.scores)


def test_cfg1_layout(cfg1):
    w = cfg1
    assert (w.B, w.H, w.d, w.L, w.C, w.Lq, w.U) == (1, 4, 128, 4096, 64, 1, 128)
    assert w.K_fixed.shape == (4, 4096, 128) and w.K_fixed.dtype == np.float16
    assert w.q.shape == (1, 4, 1, 128) and w.K_user.shape == (1, 4, 128, 128)
    assert (w.sizes.sum(1) == w.L).all()
    np.testing.assert_array_equal(w.offsets[:, 1:], np.cumsum(w.sizes, 1))
    # centroid = exact mean of the cluster's fp16 keys
    for h in range(w.H):
        for c in (0, 17, 63):
            seg = w.K_fixed[h, w.offsets[h, c]:w.offsets[h, c + 1]].astype(np.float64)
            np.testing.assert_array_equal(w.centroids[h, c], seg.mean(0).astype(np.float16))
    # keys sit next to their own centroid (sorted by cluster id)
    h = 2
    ids = np.repeat(np.arange(w.C), w.sizes[h])
    d2 = ((w.K_fixed[h].astype(np.float32)[:, None, :] - w.centroids[h].astype(np.float32)[None]) ** 2).sum(-1)
    assert (d2.argmin(1) == ids).mean() > 0.99


def test_generation_is_deterministic():
    a = wl.make_config("cfg1_tiny_decode", threads=1)
    b = wl.make_config("cfg1_tiny_decode", threads=4)
    for k in ("K_fixed", "V_fixed", "centroids", "sizes", "q", "K_user", "V_user", "q_calib"):
        np.testing.assert_array_equal(getattr(a, k), getattr(b, k))
    c = wl.make_config("cfg1_tiny_decode", seed=1)
    assert not np.array_equal(a.K_fixed, c.K_fixed)


def test_calibration_hits_keep_fraction(cfg1, oracle):
    w = cfg1
    assert w.thresh.shape == (w.H,) and (w.thresh > 0).all()
    for h in range(w.H):
        S = oracle.scores(w.q_calib[h], w.centroids[h], w.sizes[h], w.sm_scale)
        frac = ((S > w.thresh[h]) * w.sizes[h]).sum() / (wl.N_CALIB * w.L)
        assert w.keep_frac <= frac < w.keep_frac + 0.02


def test_hierarchical_workload_and_calibration(oracle):
    w = wl.make_workload("hier_small", B=1, H=2, L=8192, C=256, Lq=1, U=16, keep_frac=1 / 16, C1=16,
                         coarse_keep_frac=1 / 4)
    assert w.centroids1.shape == (2, 16, 128) and (w.sizes1.sum(1) == w.L).all()
    np.testing.assert_array_equal(w.child_offsets[0], np.arange(17) * 16)
    np.testing.assert_array_equal(w.sizes1[1, 3], w.sizes[1, 48:64].sum())
    np.testing.assert_array_equal(
        w.centroids1[0, 5], w.centroids[0, 80:96].astype(np.float64).mean(0).astype(np.float16))
    wl.calibrate(w, oracle.scores)
    kept = 0
    for h in range(w.H):
        S1 = oracle.scores(w.q_calib[h], w.centroids1[h], w.sizes1[h], w.sm_scale)
        k1 = S1 > w.thresh1[h]
        assert k1.sum() == pytest.approx(wl.N_CALIB * 16 / 4, abs=1)
        r = oracle.hier_select(np.ascontiguousarray(w.q_calib[h][:, None, :]),
                               w.centroids1[h:h + 1], w.sizes1[h:h + 1], w.child_offsets[h:h + 1], w.thresh1[h:h + 1],
                               w.centroids[h:h + 1], w.sizes[h:h + 1], w.offsets[h:h + 1], w.thresh2[h:h + 1],
                               w.sm_scale)
        frac = r["n_keys"].sum() / (wl.N_CALIB * w.L)
        assert w.keep_frac <= frac < w.keep_frac + 0.02
