"""The C-ABI library loads, exports every symbol the header declares, and validates arguments on the
host (no GPU needed: invalid calls are rejected before anything is enqueued)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def sq():
    from paper_2411_09688_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build_library()
    binding.lib()
    return binding


def test_every_declared_symbol_is_exported(sq):
    hdr = open(os.path.join(ROOT, "include", "squeezed_attention.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(sq_[a-z_0-9]+)\s*\(", hdr))
    assert {"sq_centroid_score", "sq_select", "sq_sparse_attn_decode", "sq_sparse_attn_prefill",
            "sq_hier_select"} <= declared
    L = sq.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert set(sq.EXPORTS) == declared
    assert L.sq_version() >= 100


def test_workspace_sizes(sq):
    sh = sq.make_shape(1, 32, 32768, 1024, 1, 512, 0.0884)
    assert sq.workspace_bytes(sh, sq.SQ_CALL_CENTROID_SCORE) == 0
    assert sq.workspace_bytes(sh, sq.SQ_CALL_SELECT) == 0
    a = sq.workspace_bytes(sh, sq.SQ_CALL_ATTN_DECODE)
    b = sq.workspace_bytes(sh, sq.SQ_CALL_DECODE_STEP)
    assert a > 0 and b > 0 and a % 256 == 0 and b % 256 == 0
    # partials alone: 32 rows x (2 user + 128 fixed chunks) x 132 floats
    assert a >= 32 * 130 * 132 * 4
    bad = sq.make_shape(0, 32, 32768, 1024, 1, 512, 0.0884)
    assert sq.workspace_bytes(bad, sq.SQ_CALL_ATTN_DECODE) == 0


def test_host_side_validation(sq):
    L = sq.lib()
    buf = (C.c_char * 4096)()
    p = C.cast(buf, C.c_void_p)
    aligned = C.c_void_p((p.value + 255) & ~255)
    sh = sq.make_shape(1, 2, 64, 4, 1, 0, 0.1)
    rc = L.sq_centroid_score(C.byref(sh), None, aligned, aligned, aligned, aligned, aligned, None, 0, None)
    assert rc == sq.SQ_ERR_INVALID_ARG and b"q is NULL" in L.sq_last_error()
    mis = C.c_void_p(aligned.value + 4)
    rc = L.sq_centroid_score(C.byref(sh), mis, aligned, aligned, aligned, aligned, aligned, None, 0, None)
    assert rc == sq.SQ_ERR_INVALID_ARG and b"aligned" in L.sq_last_error()
    sh64 = sq.make_shape(1, 2, 64, 4, 1, 0, 0.1, d=64)
    rc = L.sq_centroid_score(C.byref(sh64), aligned, aligned, aligned, aligned, aligned, aligned, None, 0, None)
    assert rc == sq.SQ_ERR_UNSUPPORTED
    neg = sq.make_shape(1, 2, 64, -4, 1, 0, 0.1)
    rc = L.sq_select(C.byref(neg), *([aligned] * 10), None, 0, None)
    assert rc == sq.SQ_ERR_INVALID_ARG
    pre = sq.make_shape(1, 2, 64, 4, 3, 0, 0.1)
    rc = L.sq_sparse_attn_decode(C.byref(pre), *([aligned] * 10), aligned, 1 << 30, None)
    assert rc == sq.SQ_ERR_UNSUPPORTED and b"Lq == 1" in L.sq_last_error()
    rc = L.sq_sparse_attn_decode(C.byref(sh), *([aligned] * 10), None, 0, None)
    assert rc == sq.SQ_ERR_WORKSPACE
    rc = L.sq_decode_step(C.byref(sh), *([aligned] * 13), aligned, 16, None)
    assert rc == sq.SQ_ERR_WORKSPACE and b"needed" in L.sq_last_error()


def test_host_side_validation_of_the_offline_calls(sq):
    L = sq.lib()
    buf = (C.c_char * 4096)()
    aligned = C.c_void_p((C.cast(buf, C.c_void_p).value + 255) & ~255)
    sh = sq.make_shape(1, 2, 64, 4, 1, 0, 1.0)
    assert sq.workspace_bytes(sh, sq.SQ_CALL_KMEANS_STEP) > 0 and sq.workspace_bytes(sh, sq.SQ_CALL_CALIBRATE) > 0
    rc = L.sq_kmeans_step(C.byref(sh), None, *([aligned] * 6), aligned, 1 << 30, None)
    assert rc == sq.SQ_ERR_INVALID_ARG and b"X is NULL" in L.sq_last_error()
    more = sq.make_shape(1, 2, 3, 4, 1, 0, 1.0)                  # more centres than keys
    rc = L.sq_kmeans_step(C.byref(more), *([aligned] * 7), aligned, 1 << 30, None)
    assert rc == sq.SQ_ERR_INVALID_ARG and b"more centres" in L.sq_last_error()
    rc = L.sq_kmeans_step(C.byref(sh), *([aligned] * 7), aligned, 16, None)
    assert rc == sq.SQ_ERR_WORKSPACE
    rc = L.sq_cluster_layout(C.byref(sh), aligned, aligned, aligned, aligned, aligned, aligned, aligned, aligned, None)
    assert rc == sq.SQ_ERR_INVALID_ARG and b"alias" in L.sq_last_error()
    other = C.c_void_p(aligned.value + 1024)
    rc = L.sq_cluster_layout(C.byref(sh), aligned, None, None, aligned, aligned, other, None, aligned, None)
    assert rc == sq.SQ_ERR_INVALID_ARG and b"needs perm" in L.sq_last_error()
    rc = L.sq_cluster_nest(C.byref(sh), 9, *([aligned] * 8), aligned, 1 << 30, None)
    assert rc == sq.SQ_ERR_INVALID_ARG and b"C1" in L.sq_last_error()
    rc = L.sq_calibrate_threshold(C.byref(sh), *([aligned] * 4), -1, aligned, aligned, 1 << 30, None)
    assert rc == sq.SQ_ERR_INVALID_ARG and b"negative" in L.sq_last_error()
    big = sq.make_shape(64, 2, 1 << 19, 4, 64, 0, 1.0)           # B * Lq * L = 2^31 pooled keys
    rc = L.sq_calibrate_threshold(C.byref(big), *([aligned] * 4), 5, aligned, aligned, 1 << 40, None)
    assert rc == sq.SQ_ERR_UNSUPPORTED and b"calibration queries" in L.sq_last_error()


def test_noalloc_step_rejects_oversized_shapes_on_the_host(sq):
    """sq_decode_step_noalloc checks the shape against its built-in buffer before it touches a device."""
    L = sq.lib()
    sh = sq.make_shape(4, 32, 32768, 1024, 1, 512, 0.0884)
    assert sq.workspace_bytes(sh, sq.SQ_CALL_DECODE_STEP) > sq.SQ_NOALLOC_SCRATCH_BYTES
    buf = (C.c_char * 4096)()
    p = C.c_void_p((C.cast(buf, C.c_void_p).value + 255) & ~255)
    rc = L.sq_decode_step_noalloc(C.byref(sh), p, p, p, p, p, p, p, p, p, p, None, None, None, None)
    assert rc == sq.SQ_ERR_WORKSPACE and b"built-in" in L.sq_last_error()
    fits = sq.make_shape(1, 32, 32768, 1024, 1, 512, 0.0884)
    assert sq.workspace_bytes(fits, sq.SQ_CALL_DECODE_STEP) <= sq.SQ_NOALLOC_SCRATCH_BYTES
