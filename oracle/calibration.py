"""Threshold calibration (Appendix C: one threshold chosen so that a target share of the keys is retrieved on a set of
calibration queries) -- TEST INFRASTRUCTURE ONLY, plain NumPy.

The paper states the goal (hit a target sparsity on calibration tokens), not the procedure.  Reading taken, per
head: pool the cluster scores S_i of Eq. 1 of all calibration queries, each weighing N_i keys; walk them from the
highest score down until `target_keys` keys are covered (s_k = the last score needed; a budget beyond what the
queries can retrieve at all is clamped to that); the threshold is the
geometric mean of s_k and the highest score strictly below it (half of s_k if there is none, or if that score is 0),
so that the strict rule S > T keeps exactly the walked prefix.  Scores are formed in fp32 from the fp32
(logit, maximum, normaliser) triple, the precision the selection itself works in; clusters without keys weigh nothing.

Pins: tests/test_oracle_calibration.py.
"""
from __future__ import annotations

import numpy as np


def pooled_scores(logits, row_max, denom, sizes) -> np.ndarray:
    """S [n, C] fp32 = exp(x - m) / D per calibration query (fp32 arithmetic), 0 for clusters without keys."""
    x = np.asarray(logits, dtype=np.float32)
    m = np.asarray(row_max, dtype=np.float32)[:, None]
    D = np.asarray(denom, dtype=np.float32)[:, None]
    S = (np.exp(x - m) / D).astype(np.float32)
    return np.where(np.asarray(sizes)[None, :] > 0, S, np.float32(0))


def calibrate_threshold(S, sizes, target_keys: int) -> float:
    """One head.  S [n, C] scores, sizes [C]; -> T (Python float, fp64 arithmetic on the fp32 scores)."""
    S = np.asarray(S, dtype=np.float32)
    w = np.broadcast_to(np.asarray(sizes, dtype=np.int64)[None, :], S.shape).ravel()
    s = S.ravel()
    order = np.argsort(-s, kind="stable")
    ss, cum = s[order], np.cumsum(w[order])
    k = int(np.searchsorted(cum, min(int(target_keys), int(cum[-1])), side="left"))
    s_k = float(ss[k])
    below = ss[ss < ss[k]]
    s_below = float(below.max()) if len(below) else 0.0
    if s_below <= 0.0:
        return 0.5 * s_k
    return float(np.sqrt(s_k * s_below))


def kept_keys(S, sizes, T) -> int:
    """Keys retrieved over the pooled calibration queries by the strict rule S > T."""
    S = np.asarray(S, dtype=np.float64)
    return int((np.asarray(sizes, dtype=np.int64)[None, :] * (S > T)).sum())
