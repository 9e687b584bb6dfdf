"""Pins of the threshold-calibration oracle (Appendix C): a hand example, the defining property (the budget is
met, and no higher threshold between two scores meets it), brute force over all candidate thresholds, ties."""
import numpy as np
import pytest

from oracle import calibration as cal


def test_hand_example():
    S = np.array([[0.4, 0.1], [0.3, 0.2]], np.float32)           # two queries, two clusters of 3 and 5 keys
    sizes = np.array([3, 5])
    # descending: 0.4 (3 keys), 0.3 (3), 0.2 (5), 0.1 (5); cumulative 3, 6, 11, 16
    assert cal.calibrate_threshold(S, sizes, 6) == pytest.approx(np.sqrt(np.float32(0.3) * np.float64(np.float32(0.2))))
    assert cal.calibrate_threshold(S, sizes, 7) == pytest.approx(np.sqrt(np.float32(0.2) * np.float64(np.float32(0.1))))
    assert cal.calibrate_threshold(S, sizes, 1) == pytest.approx(np.sqrt(np.float32(0.4) * np.float64(np.float32(0.3))))
    assert cal.calibrate_threshold(S, sizes, 16) == pytest.approx(0.5 * np.float32(0.1))     # nothing below: half
    assert cal.kept_keys(S, sizes, cal.calibrate_threshold(S, sizes, 7)) == 11


@pytest.mark.parametrize("seed", range(4))
def test_budget_is_met_minimally_and_matches_brute_force(seed):
    rng = np.random.default_rng(700 + seed)
    n, C = 6, 40
    S = rng.random((n, C)).astype(np.float32) ** 4
    sizes = rng.integers(0, 9, C)
    S[:, sizes == 0] = 0
    total = int(sizes.sum()) * n
    for frac in (0.05, 0.3, 0.77):
        target = int(np.ceil(frac * total))
        T = cal.calibrate_threshold(S, sizes, target)
        kept = cal.kept_keys(S, sizes, T)
        assert kept >= target
        # brute force: thresholds halfway between consecutive distinct scores; the best is the highest that meets the budget
        vals = np.unique(S.ravel())[::-1].astype(np.float64)
        cands = [np.sqrt(a * b) if b > 0 else 0.5 * a for a, b in zip(vals, list(vals[1:]) + [0.0])]
        ok = [c for c in cands if cal.kept_keys(S, sizes, c) >= target]
        assert T == pytest.approx(max(ok), rel=1e-12)
        assert kept == cal.kept_keys(S, sizes, max(ok))


def test_ties_are_dropped_or_kept_together():
    S = np.array([[0.5, 0.25, 0.25, 0.125]], np.float32)
    sizes = np.array([2, 2, 2, 2])
    T = cal.calibrate_threshold(S, sizes, 3)                     # needs one of the tied pair: both are kept
    assert T == pytest.approx(np.sqrt(0.25 * 0.125)) and cal.kept_keys(S, sizes, T) == 6


def test_pooled_scores_follow_eq1():
    rng = np.random.default_rng(710)
    x = rng.standard_normal((3, 12)).astype(np.float32)
    sizes = rng.integers(0, 5, 12)
    sizes[0] = 3
    live = sizes > 0
    m = np.where(live[None], x, -np.inf).max(1).astype(np.float32)
    D = (sizes[None] * np.exp(x.astype(np.float64) - m[:, None])).sum(1).astype(np.float32)
    S = cal.pooled_scores(x, m, D, sizes)
    np.testing.assert_allclose((S.astype(np.float64) * sizes[None]).sum(1), 1.0, rtol=1e-5)   # sum_i N_i S_i = 1
    assert (S[:, ~live] == 0).all()


def test_budget_beyond_reach_keeps_every_cluster_with_keys():
    S = np.array([[0.5, 0.0, 0.25, 0.125]], np.float32)          # cluster 1 has no keys (score forced to 0)
    sizes = np.array([2, 0, 2, 2])
    T = cal.calibrate_threshold(S, sizes, 100)                   # clamped to 6: the last score needed is 0.125
    assert T == pytest.approx(0.5 * 0.125) and cal.kept_keys(S, sizes, T) == 6
