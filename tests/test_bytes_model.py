"""The byte model against the KV budgets the paper prints."""
import numpy as np
import pytest

from golden_io import read_records
from paper_2411_09688_amd import bytes_model as bm


def test_kv_budget_matches_paper_table():
    g = read_records("kv_budget_table.txt")
    c = g["one_level"]["centroid_frac"][0]
    for s, b in zip(g["one_level"]["sparsity"], g["one_level"]["budget"]):
        assert bm.kv_budget(s, c) == pytest.approx(b, abs=1e-12)
    assert bm.centroid_overhead(c)[1] == pytest.approx(0.025)
    c1, c2 = g["two_level"]["centroid_fracs"]
    stored, loaded = bm.centroid_overhead(c1, c2, g["two_level"]["coarse_keep"][0])
    assert (stored, loaded) == pytest.approx(tuple(g["two_level"]["stored_loaded"]))


def test_decode_step_bytes_config2_nominal():
    # config 2 at exactly 1/8 kept: 8 MiB centroids + 64 MiB selected K/V + 8 MiB dense K/V (+ metadata)
    b = bm.decode_step_bytes(H=32, C=1024, d=128, U=512, B=1, n_keys_per_row=np.full(32, 4096))
    assert b["centroid"] == 8 << 20 and b["selected_kv"] == 64 << 20 and b["dense_kv"] == 8 << 20
    assert b["total"] - (80 << 20) < (1 << 19)
