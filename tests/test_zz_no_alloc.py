"""GPU: the decode step that takes no workspace and allocates nothing (sq_decode_step_noalloc) against sq_decode_step
on the same inputs -- two calls in a row, the second on a smaller problem, which finds the first call's state in the
library's built-in buffer."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2411_09688_amd import workload as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sq():
    from paper_2411_09688_amd import binding
    binding.lib()
    return binding


def both_steps(sq, w):
    P = sq.upload(w)
    sh = P.shape
    ref = dict(out=torch.full_like(P.out, 7.0), lse=torch.zeros_like(P.lse), mask=torch.zeros_like(P.keep_mask),
               nk=torch.zeros_like(P.n_keys))
    got = {k: v.clone() for k, v in ref.items()}
    ws = sq.workspace(sh, sq.SQ_CALL_DECODE_STEP, P.q.device)
    sq.sq_decode_step(sh, P.q, P.centroids, P.sizes, P.offsets, P.thresh, P.K_fixed, P.V_fixed, P.K_user, P.V_user,
                      ref["out"], ref["lse"], ref["mask"], ref["nk"], ws)
    torch.cuda.synchronize()
    sq.sq_decode_step_noalloc(sh, P.q, P.centroids, P.sizes, P.offsets, P.thresh, P.K_fixed, P.V_fixed, P.K_user,
                              P.V_user, got["out"], got["lse"], got["mask"], got["nk"])
    torch.cuda.synchronize()
    # integer results bit for bit; attention to the bar of the parity tests (the two calls may split the keys over
    # workgroups differently: fp32 partial sums regrouped, fp16 output)
    assert torch.equal(got["mask"], ref["mask"]) and torch.equal(got["nk"], ref["nk"])
    assert ref["nk"].sum().item() > 0
    err = (got["out"].float() - ref["out"].float()).abs().max().item()
    assert err <= 2e-3, err
    torch.testing.assert_close(got["lse"], ref["lse"], atol=1e-4, rtol=1e-5)
    return err


def test_noalloc_step_twice_second_smaller(sq, oracle):
    big = wl.calibrate(wl.make_workload("noalloc_big", B=1, H=32, L=32768, C=1024, Lq=1, U=512, keep_frac=0.125, seed=41,
                                        threads=8), oracle.scores)
    assert sq.workspace_bytes(sq.upload(big).shape, sq.SQ_CALL_DECODE_STEP) <= sq.SQ_NOALLOC_SCRATCH_BYTES
    small = wl.calibrate(wl.make_workload("noalloc_small", B=2, H=3, L=3000, C=100, Lq=1, U=300, keep_frac=0.5, seed=42,
                                          threads=2), oracle.scores)
    print("no-alloc step, large then small:", both_steps(sq, big), both_steps(sq, small), flush=True)


def test_noalloc_step_rejects_shapes_beyond_its_buffer(sq):
    sh = sq.make_shape(4, 32, 32768, 1024, 1, 512, 0.0884)      # four sequences: needs more than the built-in buffer
    assert sq.workspace_bytes(sh, sq.SQ_CALL_DECODE_STEP) > sq.SQ_NOALLOC_SCRATCH_BYTES
    dummy = torch.zeros(64, dtype=torch.float16, device="cuda:0")
    p = C.c_void_p(dummy.data_ptr())
    rc = sq.lib().sq_decode_step_noalloc(C.byref(sh), p, p, p, p, p, p, p, p, p, p, None, None, None, None)
    assert rc == sq.SQ_ERR_WORKSPACE and b"built-in" in sq.lib().sq_last_error()
