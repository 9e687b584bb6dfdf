"""Seeded random shapes through the step entry points, checked with the same helpers (and so the same bars) as the
hand-picked cases of the other GPU test modules: every draw is a shape nobody chose, which is where tile boundaries,
ragged tails and empty pieces that the fixed cases miss would show."""
import numpy as np
import pytest

import test_gpu_decode as td
import test_gpu_gqa as tg
import test_gpu_hier as th
import test_gpu_prefill as tp
from gpu_util import oracle_one_level
from paper_2411_09688_amd import workload as wl

pytestmark = pytest.mark.gpu

USER_KEYS = [0, 1, 5, 127, 128, 129, 300, 513, 1000]      # around the 128-key chunk and block boundaries


@pytest.fixture(scope="module")
def sq():
    from paper_2411_09688_amd import binding
    binding.lib()
    return binding


@pytest.mark.parametrize("seed", [11, 12])
def test_decode_step_random_shapes(sq, oracle, seed):
    rng = np.random.default_rng(seed)
    for it in range(8):
        L = int(rng.integers(200, 5000))
        case = dict(B=int(rng.integers(1, 8)), H=int(rng.integers(1, 4)), L=L, C=int(rng.integers(1, min(L, 2300))),
                    U=int(rng.choice(USER_KEYS)), keep_frac=float(rng.uniform(0.05, 0.9)))
        w = wl.calibrate(wl.make_workload("rnd_decode", Lq=1, seed=1000 * seed + it, threads=2, **case), oracle.scores)
        P = sq.upload(w)
        td.run_separate(sq, w, P)
        td.compare_decode(oracle, w, P, oracle_one_level(oracle, w), f"random decode {case}")
        td.fused_matches(sq, w, P)


@pytest.mark.parametrize("seed", [21])
def test_two_level_step_random_shapes(sq, oracle, seed):
    rng = np.random.default_rng(seed)
    for it in range(8):
        C1 = int(rng.integers(2, 40))
        C = C1 * int(rng.integers(1, 70))                  # up to 2760 fine clusters: candidate rows of several steps
        L = int(rng.integers(max(C, 300), max(C, 300) * 6))
        case = dict(B=int(rng.integers(1, 3)), H=int(rng.integers(1, 3)), L=L, C=C, Lq=1, U=int(rng.choice(USER_KEYS)),
                    keep_frac=float(rng.uniform(0.05, 0.6)), C1=C1, coarse_keep_frac=float(rng.uniform(0.1, 0.9)))
        w = wl.make_workload("rnd_hier", seed=1000 * seed + it, threads=2, **case)
        wl.calibrate(w, oracle.scores)
        th.hier_decode_and_compare(sq, oracle, w, f"random two-level {case}")


@pytest.mark.parametrize("seed", [31])
def test_shared_context_and_grouped_query_random_shapes(sq, oracle, seed):
    rng = np.random.default_rng(seed)
    for it in range(5):
        L = int(rng.integers(300, 5000))
        case = dict(B=int(rng.integers(8, 21)), H=int(rng.integers(1, 3)), L=L, C=min(int(rng.integers(2, 300)), L),
                    U=int(rng.choice(USER_KEYS)), keep_frac=float(rng.uniform(0.1, 0.7)))
        td.test_shared_context_step_against_oracle(sq, oracle, case)
        gcase = dict(G=int(rng.choice([1, 2, 4, 8, 16])), B=int(rng.integers(1, 5)), H=int(rng.integers(1, 3)),
                     L=int(rng.integers(300, 4000)), C=int(rng.integers(2, 200)), U=int(rng.choice(USER_KEYS)),
                     keep_frac=float(rng.uniform(0.1, 0.7)))
        tg.test_gqa_step_against_oracle(sq, gcase)
        tg.test_gqa_mean_step_against_oracle(sq, gcase)


@pytest.mark.parametrize("seed", [41, 42, 43])
def test_prefill_steps_random_shapes(sq, oracle, seed):
    rng = np.random.default_rng(seed)
    for it in range(6):
        Lq = int(rng.choice([1, 15, 16, 17, 63, 64, 65, 127, 128, 129, 200, 257, 300]))
        causal = bool(rng.integers(0, 2))
        U = int(rng.choice([Lq, max(Lq, 64), Lq + 37])) if causal else int(rng.choice([0, 1, 63, 64, 65, 130, 300]))
        L = int(rng.integers(200, 3000))
        case = dict(B=int(rng.integers(1, 3)), H=int(rng.integers(1, 3)), L=L, C=int(rng.integers(1, min(L, 400))), Lq=Lq,
                    U=U, keep_frac=float(rng.uniform(0.1, 0.8)), causal_user=causal)
        tp.test_prefill_small(sq, oracle, case)
        tp.test_prefill_step_small(sq, oracle, case)
        tp.test_prefill_mean_step_small(sq, oracle, case)
