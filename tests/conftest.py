import os
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run through the C-ABI library)")


def pytest_collection_modifyitems(config, items):
    """GPU tests are skipped on a machine without a GPU instead of failing at import time."""
    try:
        import torch
        have_gpu = torch.cuda.is_available()
    except Exception:  # pragma: no cover
        have_gpu = False
    if have_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU in this process")
    for it in items:
        if "gpu" in it.keywords:
            it.add_marker(skip)


@pytest.fixture(scope="session")
def oracle():
    import oracle as o
    o.build()
    return o


def random_problem(rng, H, C, d, nq, max_size=5, zero_frac=0.0):
    """Small random one-level problem with fp16-representable values (not the mixture generator)."""
    cent = (rng.standard_normal((H, C, d)) * 0.7).astype(np.float16)
    sizes = rng.integers(1, max_size + 1, size=(H, C)).astype(np.int32)
    if zero_frac:
        sizes[rng.random((H, C)) < zero_frac] = 0
    offsets = np.zeros((H, C + 1), np.int32)
    offsets[:, 1:] = np.cumsum(sizes, axis=1)
    q = (rng.standard_normal((1, H, nq, d)) * 0.9).astype(np.float16)
    return cent, sizes, offsets, q
