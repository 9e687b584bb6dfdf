"""Thin Python binding of the C-ABI library (`include/squeezed_attention.h`).

Argument marshalling only: every function checks dtypes / contiguity of the torch tensors it is
given, passes their device pointers to the entry point of the same name, and raises on a non-zero
status.  torch supplies device memory and the current stream; nothing is computed here, and there
is no fallback: if the HIP library has not been built, importing it raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libsqueezed_attention.so")

SQ_OK, SQ_ERR_INVALID_ARG, SQ_ERR_UNSUPPORTED, SQ_ERR_WORKSPACE, SQ_ERR_HIP = 0, -1, -2, -3, -4
(SQ_CALL_CENTROID_SCORE, SQ_CALL_SELECT, SQ_CALL_ATTN_DECODE, SQ_CALL_ATTN_PREFILL, SQ_CALL_HIER_SELECT,
 SQ_CALL_DECODE_STEP, SQ_CALL_HIER_DECODE_STEP, SQ_CALL_SELECT_MEAN, SQ_CALL_ATTN_PREFILL_SHARED,
 SQ_CALL_PREFILL_STEP, SQ_CALL_PREFILL_MEAN_STEP, SQ_CALL_GQA_DECODE_STEP, SQ_CALL_MULTILEVEL_SELECT,
 SQ_CALL_MULTILEVEL_DECODE_STEP, SQ_CALL_KMEANS_STEP, SQ_CALL_CALIBRATE, SQ_CALL_HIER_PREFILL_MEAN_STEP, SQ_CALL_GQA_MEAN_DECODE_STEP, SQ_CALL_HIER_PREFILL_STEP) = range(19)
SQ_MAX_LEVELS = 4

EXPORTS = ("sq_workspace_bytes", "sq_last_error", "sq_version", "sq_centroid_score", "sq_select",
           "sq_sparse_attn_decode", "sq_sparse_attn_prefill", "sq_hier_select", "sq_decode_step",
           "sq_hier_decode_step", "sq_decode_step_noalloc", "sq_select_mean", "sq_sparse_attn_prefill_shared", "sq_prefill_step",
           "sq_prefill_mean_step", "sq_gqa_decode_step", "sq_multilevel_select", "sq_multilevel_decode_step",
           "sq_kmeans_normalize", "sq_kmeans_step", "sq_cluster_layout", "sq_cluster_nest", "sq_calibrate_threshold", "sq_hier_prefill_mean_step", "sq_hier_prefill_step", "sq_gqa_mean_decode_step", "sq_profile_begin",
           "sq_profile_end", "sq_probe_stream_read")


class SqShape(C.Structure):
    _fields_ = [("B", C.c_int32), ("H", C.c_int32), ("d", C.c_int32), ("L", C.c_int32), ("C", C.c_int32),
                ("Lq", C.c_int32), ("U", C.c_int32), ("sm_scale", C.c_float), ("causal_user", C.c_int32)]


class SqLevel(C.Structure):
    _fields_ = [("C", C.c_int32), ("centroids", C.c_void_p), ("sizes", C.c_void_p), ("child_offsets", C.c_void_p),
                ("thresh", C.c_void_p)]


class SqError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"squeezed_attention error {code}: {msg}")
        self.code = code


_lib = None


def lib() -> C.CDLL:
    """The loaded shared library; raises if it has not been built (no fallback path exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2411_09688_amd.build` "
                              "(or __graft_entry__.build())")
        L = C.CDLL(LIB_PATH)
        L.sq_workspace_bytes.restype = C.c_size_t
        L.sq_workspace_bytes.argtypes = [C.POINTER(SqShape), C.c_int]
        L.sq_last_error.restype = C.c_char_p
        L.sq_version.restype = C.c_int
        vp, sz = C.c_void_p, C.c_size_t
        sp = C.POINTER(SqShape)
        L.sq_centroid_score.argtypes = [sp] + [vp] * 6 + [vp, sz, vp]
        L.sq_select.argtypes = [sp] + [vp] * 10 + [vp, sz, vp]
        L.sq_sparse_attn_decode.argtypes = [sp] + [vp] * 10 + [vp, sz, vp]
        L.sq_sparse_attn_prefill.argtypes = [sp] + [vp] * 9 + [vp, sz, vp]
        L.sq_hier_select.argtypes = [sp, C.c_int32] + [vp] * 14 + [vp, sz, vp]
        L.sq_decode_step.argtypes = [sp] + [vp] * 13 + [vp, sz, vp]
        L.sq_decode_step_noalloc.argtypes = [sp] + [vp] * 13 + [vp]
        L.sq_hier_decode_step.argtypes = [sp, C.c_int32] + [vp] * 17 + [vp, sz, vp]
        L.sq_hier_prefill_step.argtypes = [sp, C.c_int32] + [vp] * 17 + [vp, sz, vp]
        L.sq_hier_prefill_mean_step.argtypes = [sp, C.c_int32] + [vp] * 17 + [vp, sz, vp]
        L.sq_gqa_mean_decode_step.argtypes = [sp, C.c_int32] + [vp] * 13 + [vp, sz, vp]
        L.sq_gqa_decode_step.argtypes = [sp, C.c_int32] + [vp] * 13 + [vp, sz, vp]
        lp = C.POINTER(SqLevel)
        L.sq_multilevel_select.argtypes = [sp, C.c_int32, lp, vp, C.POINTER(vp)] + [vp] * 3 + [vp, sz, vp]
        L.sq_multilevel_decode_step.argtypes = [sp, C.c_int32, lp] + [vp] * 9 + [vp, sz, vp]
        L.sq_kmeans_normalize.argtypes = [sp, vp, vp, vp]
        L.sq_kmeans_step.argtypes = [sp] + [vp] * 7 + [vp, sz, vp]
        L.sq_cluster_layout.argtypes = [sp] + [vp] * 8 + [vp]
        L.sq_cluster_nest.argtypes = [sp, C.c_int32] + [vp] * 8 + [vp, sz, vp]
        L.sq_calibrate_threshold.argtypes = [sp] + [vp] * 4 + [C.c_int64, vp] + [vp, sz, vp]
        L.sq_probe_stream_read.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_int, C.c_void_p]
        L.sq_profile_begin.argtypes = [C.c_int]
        L.sq_profile_end.argtypes = [C.POINTER(C.c_float)] * 3
        for name in EXPORTS[3:]:
            getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def make_shape(B, H, L, Cn, Lq, U, sm_scale, causal_user=False, d=128) -> SqShape:
    return SqShape(B, H, d, L, Cn, Lq, U, float(sm_scale), int(bool(causal_user)))


def workspace_bytes(shape: SqShape, which: int) -> int:
    return int(lib().sq_workspace_bytes(C.byref(shape), which))


_ws_cache: dict = {}


def workspace(shape: SqShape, which: int, device) -> Optional[torch.Tensor]:
    """A cached device byte buffer large enough for the call (torch's allocator aligns to 256 B or more)."""
    n = workspace_bytes(shape, which)
    if n == 0:
        return None
    key = (str(device), which)
    buf = _ws_cache.get(key)
    if buf is None or buf.numel() < n:
        buf = torch.empty(n, dtype=torch.uint8, device=device)
        _ws_cache[key] = buf
    return buf


def _ptr(t: Optional[torch.Tensor], dtype=None, name="tensor"):
    if t is None:
        return None
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"{name} must be {dtype}, got {t.dtype}")
    return C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _check(rc: int):
    if rc != SQ_OK:
        raise SqError(rc, lib().sq_last_error().decode())


def _ws_args(ws: Optional[torch.Tensor]):
    return (None, 0) if ws is None else (C.c_void_p(ws.data_ptr()), ws.numel() * ws.element_size())


F16, F32, I32 = torch.float16, torch.float32, torch.int32


def sq_centroid_score(shape, q, centroids, sizes, logits, row_max, denom, ws=None, stream=None):
    _check(lib().sq_centroid_score(C.byref(shape), _ptr(q, F16, "q"), _ptr(centroids, F16, "centroids"),
                                   _ptr(sizes, I32, "sizes"), _ptr(logits, F32, "logits"),
                                   _ptr(row_max, F32, "row_max"), _ptr(denom, F32, "denom"), *_ws_args(ws),
                                   _stream(stream)))


def sq_select(shape, logits, row_max, denom, thresh, sizes, offsets, keep_mask, ranges, n_ranges, n_keys, ws=None,
              stream=None):
    _check(lib().sq_select(C.byref(shape), _ptr(logits, F32, "logits"), _ptr(row_max, F32, "row_max"),
                           _ptr(denom, F32, "denom"), _ptr(thresh, F32, "thresh"), _ptr(sizes, I32, "sizes"),
                           _ptr(offsets, I32, "offsets"), _ptr(keep_mask, I32, "keep_mask"),
                           _ptr(ranges, I32, "ranges"), _ptr(n_ranges, I32, "n_ranges"), _ptr(n_keys, I32, "n_keys"),
                           *_ws_args(ws), _stream(stream)))


def sq_sparse_attn_decode(shape, q, K_fixed, V_fixed, ranges, n_ranges, n_keys, K_user, V_user, out, lse, ws,
                          stream=None):
    _check(lib().sq_sparse_attn_decode(C.byref(shape), _ptr(q, F16, "q"), _ptr(K_fixed, F16, "K_fixed"),
                                       _ptr(V_fixed, F16, "V_fixed"), _ptr(ranges, I32, "ranges"),
                                       _ptr(n_ranges, I32, "n_ranges"), _ptr(n_keys, I32, "n_keys"),
                                       _ptr(K_user, F16, "K_user"), _ptr(V_user, F16, "V_user"),
                                       _ptr(out, F16, "out"), _ptr(lse, F32, "lse"), *_ws_args(ws), _stream(stream)))


def sq_sparse_attn_prefill(shape, q, K_fixed, V_fixed, offsets, keep_mask, K_user, V_user, out, lse, ws, stream=None):
    _check(lib().sq_sparse_attn_prefill(C.byref(shape), _ptr(q, F16, "q"), _ptr(K_fixed, F16, "K_fixed"),
                                        _ptr(V_fixed, F16, "V_fixed"), _ptr(offsets, I32, "offsets"),
                                        _ptr(keep_mask, I32, "keep_mask"), _ptr(K_user, F16, "K_user"),
                                        _ptr(V_user, F16, "V_user"), _ptr(out, F16, "out"), _ptr(lse, F32, "lse"),
                                        *_ws_args(ws), _stream(stream)))


def sq_select_mean(shape, logits, row_max, denom, thresh, sizes, offsets, keep_mask, ranges, n_ranges, n_keys, ws,
                   stream=None):
    _check(lib().sq_select_mean(C.byref(shape), _ptr(logits, F32, "logits"), _ptr(row_max, F32, "row_max"),
                                _ptr(denom, F32, "denom"), _ptr(thresh, F32, "thresh"), _ptr(sizes, I32, "sizes"),
                                _ptr(offsets, I32, "offsets"), _ptr(keep_mask, I32, "keep_mask"),
                                _ptr(ranges, I32, "ranges"), _ptr(n_ranges, I32, "n_ranges"),
                                _ptr(n_keys, I32, "n_keys"), *_ws_args(ws), _stream(stream)))


def sq_sparse_attn_prefill_shared(shape, q, K_fixed, V_fixed, ranges, n_ranges, n_keys, K_user, V_user, out, lse, ws,
                                  stream=None):
    _check(lib().sq_sparse_attn_prefill_shared(C.byref(shape), _ptr(q, F16, "q"), _ptr(K_fixed, F16, "K_fixed"),
                                               _ptr(V_fixed, F16, "V_fixed"), _ptr(ranges, I32, "ranges"),
                                               _ptr(n_ranges, I32, "n_ranges"), _ptr(n_keys, I32, "n_keys"),
                                               _ptr(K_user, F16, "K_user"), _ptr(V_user, F16, "V_user"),
                                               _ptr(out, F16, "out"), _ptr(lse, F32, "lse"), *_ws_args(ws),
                                               _stream(stream)))


def _prefill_step(fn, shape, q, centroids, sizes, offsets, thresh, K_fixed, V_fixed, K_user, V_user, out, lse, keep_mask,
                  n_keys, ws, stream):
    _check(fn(C.byref(shape), _ptr(q, F16, "q"), _ptr(centroids, F16, "centroids"), _ptr(sizes, I32, "sizes"),
              _ptr(offsets, I32, "offsets"), _ptr(thresh, F32, "thresh"), _ptr(K_fixed, F16, "K_fixed"),
              _ptr(V_fixed, F16, "V_fixed"), _ptr(K_user, F16, "K_user"), _ptr(V_user, F16, "V_user"),
              _ptr(out, F16, "out"), _ptr(lse, F32, "lse"), _ptr(keep_mask, I32, "keep_mask"),
              _ptr(n_keys, I32, "n_keys"), *_ws_args(ws), _stream(stream)))


def sq_prefill_step(shape, q, centroids, sizes, offsets, thresh, K_fixed, V_fixed, K_user, V_user, out, lse, keep_mask,
                    n_keys, ws, stream=None):
    _prefill_step(lib().sq_prefill_step, shape, q, centroids, sizes, offsets, thresh, K_fixed, V_fixed, K_user, V_user,
                  out, lse, keep_mask, n_keys, ws, stream)


def sq_prefill_mean_step(shape, q, centroids, sizes, offsets, thresh, K_fixed, V_fixed, K_user, V_user, out, lse,
                         keep_mask, n_keys, ws, stream=None):
    _prefill_step(lib().sq_prefill_mean_step, shape, q, centroids, sizes, offsets, thresh, K_fixed, V_fixed, K_user,
                  V_user, out, lse, keep_mask, n_keys, ws, stream)


def sq_hier_select(shape, C1, q, centroids1, sizes1, child_offsets, thresh1, centroids2, sizes2, offsets2, thresh2,
                   keep_mask1, keep_mask2, ranges, n_ranges, n_keys, ws, stream=None):
    _check(lib().sq_hier_select(C.byref(shape), int(C1), _ptr(q, F16, "q"), _ptr(centroids1, F16, "centroids1"),
                                _ptr(sizes1, I32, "sizes1"), _ptr(child_offsets, I32, "child_offsets"),
                                _ptr(thresh1, F32, "thresh1"), _ptr(centroids2, F16, "centroids2"),
                                _ptr(sizes2, I32, "sizes2"), _ptr(offsets2, I32, "offsets2"),
                                _ptr(thresh2, F32, "thresh2"), _ptr(keep_mask1, I32, "keep_mask1"),
                                _ptr(keep_mask2, I32, "keep_mask2"), _ptr(ranges, I32, "ranges"),
                                _ptr(n_ranges, I32, "n_ranges"), _ptr(n_keys, I32, "n_keys"), *_ws_args(ws),
                                _stream(stream)))


def sq_decode_step(shape, q, centroids, sizes, offsets, thresh, K_fixed, V_fixed, K_user, V_user, out, lse, keep_mask,
                   n_keys, ws, stream=None):
    _check(lib().sq_decode_step(C.byref(shape), _ptr(q, F16, "q"), _ptr(centroids, F16, "centroids"),
                                _ptr(sizes, I32, "sizes"), _ptr(offsets, I32, "offsets"), _ptr(thresh, F32, "thresh"),
                                _ptr(K_fixed, F16, "K_fixed"), _ptr(V_fixed, F16, "V_fixed"),
                                _ptr(K_user, F16, "K_user"), _ptr(V_user, F16, "V_user"), _ptr(out, F16, "out"),
                                _ptr(lse, F32, "lse"), _ptr(keep_mask, I32, "keep_mask"), _ptr(n_keys, I32, "n_keys"),
                                *_ws_args(ws), _stream(stream)))


SQ_NOALLOC_SCRATCH_BYTES = 16 << 20


def sq_decode_step_noalloc(shape, q, centroids, sizes, offsets, thresh, K_fixed, V_fixed, K_user, V_user, out, lse,
                           keep_mask, n_keys, stream=None):
    _check(lib().sq_decode_step_noalloc(C.byref(shape), _ptr(q, F16, "q"), _ptr(centroids, F16, "centroids"),
                                        _ptr(sizes, I32, "sizes"), _ptr(offsets, I32, "offsets"),
                                        _ptr(thresh, F32, "thresh"), _ptr(K_fixed, F16, "K_fixed"),
                                        _ptr(V_fixed, F16, "V_fixed"), _ptr(K_user, F16, "K_user"),
                                        _ptr(V_user, F16, "V_user"), _ptr(out, F16, "out"), _ptr(lse, F32, "lse"),
                                        _ptr(keep_mask, I32, "keep_mask"), _ptr(n_keys, I32, "n_keys"),
                                        _stream(stream)))


def sq_gqa_decode_step(shape, G, q, centroids, sizes, offsets, thresh, K_fixed, V_fixed, K_user, V_user, out, lse,
                       keep_mask, n_keys, ws, stream=None):
    _check(lib().sq_gqa_decode_step(C.byref(shape), int(G), _ptr(q, F16, "q"), _ptr(centroids, F16, "centroids"),
                                    _ptr(sizes, I32, "sizes"), _ptr(offsets, I32, "offsets"),
                                    _ptr(thresh, F32, "thresh"), _ptr(K_fixed, F16, "K_fixed"),
                                    _ptr(V_fixed, F16, "V_fixed"), _ptr(K_user, F16, "K_user"),
                                    _ptr(V_user, F16, "V_user"), _ptr(out, F16, "out"), _ptr(lse, F32, "lse"),
                                    _ptr(keep_mask, I32, "keep_mask"), _ptr(n_keys, I32, "n_keys"), *_ws_args(ws),
                                    _stream(stream)))


def sq_gqa_mean_decode_step(shape, G, q, centroids, sizes, offsets, thresh, K_fixed, V_fixed, K_user, V_user, out, lse,
                            keep_mask, n_keys, ws, stream=None):
    _check(lib().sq_gqa_mean_decode_step(C.byref(shape), int(G), _ptr(q, F16, "q"), _ptr(centroids, F16, "centroids"),
                                         _ptr(sizes, I32, "sizes"), _ptr(offsets, I32, "offsets"),
                                         _ptr(thresh, F32, "thresh"), _ptr(K_fixed, F16, "K_fixed"),
                                         _ptr(V_fixed, F16, "V_fixed"), _ptr(K_user, F16, "K_user"),
                                         _ptr(V_user, F16, "V_user"), _ptr(out, F16, "out"), _ptr(lse, F32, "lse"),
                                         _ptr(keep_mask, I32, "keep_mask"), _ptr(n_keys, I32, "n_keys"), *_ws_args(ws),
                                         _stream(stream)))


def _levels(levels):
    """levels: list of (centroids f16 [H,C,d], sizes i32 [H,C], child_offsets i32 [H,C+1], thresh f32 [H]) tensors."""
    arr = (SqLevel * len(levels))()
    for k, (cen, siz, cof, thr) in enumerate(levels):
        arr[k] = SqLevel(int(cen.shape[1]), _ptr(cen, F16, "centroids"), _ptr(siz, I32, "sizes"),
                         _ptr(cof, I32, "child_offsets"), _ptr(thr, F32, "thresh"))
    return arr


def sq_multilevel_select(shape, levels, q, keep_masks, ranges, n_ranges, n_keys, ws, stream=None):
    """keep_masks: None, or a list (one entry per level) of int32 tensors / None."""
    arr = _levels(levels)
    masks = None
    if keep_masks is not None:
        masks = (C.c_void_p * len(levels))(*[_ptr(m, I32, "keep_mask") for m in keep_masks])
    _check(lib().sq_multilevel_select(C.byref(shape), len(levels), arr, _ptr(q, F16, "q"), masks,
                                      _ptr(ranges, I32, "ranges"), _ptr(n_ranges, I32, "n_ranges"),
                                      _ptr(n_keys, I32, "n_keys"), *_ws_args(ws), _stream(stream)))


def sq_multilevel_decode_step(shape, levels, q, K_fixed, V_fixed, K_user, V_user, out, lse, keep_mask, n_keys, ws,
                              stream=None):
    arr = _levels(levels)
    _check(lib().sq_multilevel_decode_step(C.byref(shape), len(levels), arr, _ptr(q, F16, "q"),
                                           _ptr(K_fixed, F16, "K_fixed"), _ptr(V_fixed, F16, "V_fixed"),
                                           _ptr(K_user, F16, "K_user"), _ptr(V_user, F16, "V_user"),
                                           _ptr(out, F16, "out"), _ptr(lse, F32, "lse"),
                                           _ptr(keep_mask, I32, "keep_mask"), _ptr(n_keys, I32, "n_keys"),
                                           *_ws_args(ws), _stream(stream)))


def sq_hier_decode_step(shape, C1, q, centroids1, sizes1, child_offsets, thresh1, centroids2, sizes2, offsets2,
                        thresh2, K_fixed, V_fixed, K_user, V_user, out, lse, keep_mask2, n_keys, ws, stream=None):
    _check(lib().sq_hier_decode_step(
        C.byref(shape), int(C1), _ptr(q, F16, "q"), _ptr(centroids1, F16, "centroids1"), _ptr(sizes1, I32, "sizes1"),
        _ptr(child_offsets, I32, "child_offsets"), _ptr(thresh1, F32, "thresh1"),
        _ptr(centroids2, F16, "centroids2"), _ptr(sizes2, I32, "sizes2"), _ptr(offsets2, I32, "offsets2"),
        _ptr(thresh2, F32, "thresh2"), _ptr(K_fixed, F16, "K_fixed"), _ptr(V_fixed, F16, "V_fixed"),
        _ptr(K_user, F16, "K_user"), _ptr(V_user, F16, "V_user"), _ptr(out, F16, "out"), _ptr(lse, F32, "lse"),
        _ptr(keep_mask2, I32, "keep_mask2"), _ptr(n_keys, I32, "n_keys"), *_ws_args(ws), _stream(stream)))


def sq_kmeans_normalize(shape, K, X, stream=None):
    _check(lib().sq_kmeans_normalize(C.byref(shape), _ptr(K, F16, "K"), _ptr(X, F16, "X"), _stream(stream)))


def sq_kmeans_step(shape, X, centers_in, centers_out, assign, sizes, offsets, perm, ws, stream=None):
    _check(lib().sq_kmeans_step(C.byref(shape), _ptr(X, F16, "X"), _ptr(centers_in, F16, "centers_in"),
                                _ptr(centers_out, F16, "centers_out"), _ptr(assign, I32, "assign"),
                                _ptr(sizes, I32, "sizes"), _ptr(offsets, I32, "offsets"), _ptr(perm, I32, "perm"),
                                *_ws_args(ws), _stream(stream)))


def sq_cluster_layout(shape, K, V, perm, sizes, offsets, K_sorted, V_sorted, centroids, stream=None):
    _check(lib().sq_cluster_layout(C.byref(shape), _ptr(K, F16, "K"), _ptr(V, F16, "V"), _ptr(perm, I32, "perm"),
                                   _ptr(sizes, I32, "sizes"), _ptr(offsets, I32, "offsets"),
                                   _ptr(K_sorted, F16, "K_sorted"), _ptr(V_sorted, F16, "V_sorted"),
                                   _ptr(centroids, F16, "centroids"), _stream(stream)))


def sq_cluster_nest(shape, C1, assign_fine, perm_coarse, child_offsets, assign_new, sizes, offsets, perm, sizes_coarse,
                    ws, stream=None):
    _check(lib().sq_cluster_nest(C.byref(shape), int(C1), _ptr(assign_fine, I32, "assign_fine"),
                                 _ptr(perm_coarse, I32, "perm_coarse"), _ptr(child_offsets, I32, "child_offsets"),
                                 _ptr(assign_new, I32, "assign_new"), _ptr(sizes, I32, "sizes"),
                                 _ptr(offsets, I32, "offsets"), _ptr(perm, I32, "perm"),
                                 _ptr(sizes_coarse, I32, "sizes_coarse"), *_ws_args(ws), _stream(stream)))


def sq_calibrate_threshold(shape, logits, row_max, denom, sizes, target_keys, thresh, ws, stream=None):
    _check(lib().sq_calibrate_threshold(C.byref(shape), _ptr(logits, F32, "logits"), _ptr(row_max, F32, "row_max"),
                                        _ptr(denom, F32, "denom"), _ptr(sizes, I32, "sizes"), int(target_keys),
                                        _ptr(thresh, F32, "thresh"), *_ws_args(ws), _stream(stream)))


def _hier_prefill(fn, shape, C1, q, centroids1, sizes1, child_offsets, thresh1, centroids2, sizes2, offsets2, thresh2,
                  K_fixed, V_fixed, K_user, V_user, out, lse, keep_mask2, n_keys, ws, stream):
    _check(fn(
        C.byref(shape), int(C1), _ptr(q, F16, "q"), _ptr(centroids1, F16, "centroids1"), _ptr(sizes1, I32, "sizes1"),
        _ptr(child_offsets, I32, "child_offsets"), _ptr(thresh1, F32, "thresh1"),
        _ptr(centroids2, F16, "centroids2"), _ptr(sizes2, I32, "sizes2"), _ptr(offsets2, I32, "offsets2"),
        _ptr(thresh2, F32, "thresh2"), _ptr(K_fixed, F16, "K_fixed"), _ptr(V_fixed, F16, "V_fixed"),
        _ptr(K_user, F16, "K_user"), _ptr(V_user, F16, "V_user"), _ptr(out, F16, "out"), _ptr(lse, F32, "lse"),
        _ptr(keep_mask2, I32, "keep_mask2"), _ptr(n_keys, I32, "n_keys"), *_ws_args(ws), _stream(stream)))


def sq_hier_prefill_step(shape, C1, q, centroids1, sizes1, child_offsets, thresh1, centroids2, sizes2, offsets2, thresh2,
                         K_fixed, V_fixed, K_user, V_user, out, lse, keep_mask2, n_keys, ws, stream=None):
    """Per-token selection: keep_mask2 [B,H,Lq,W], n_keys [B,H,Lq]."""
    _hier_prefill(lib().sq_hier_prefill_step, shape, C1, q, centroids1, sizes1, child_offsets, thresh1, centroids2,
                  sizes2, offsets2, thresh2, K_fixed, V_fixed, K_user, V_user, out, lse, keep_mask2, n_keys, ws, stream)


def sq_hier_prefill_mean_step(shape, C1, q, centroids1, sizes1, child_offsets, thresh1, centroids2, sizes2, offsets2,
                              thresh2, K_fixed, V_fixed, K_user, V_user, out, lse, keep_mask2, n_keys, ws, stream=None):
    """One kept set per (sequence, head): keep_mask2 [B,H,W], n_keys [B,H]."""
    _hier_prefill(lib().sq_hier_prefill_mean_step, shape, C1, q, centroids1, sizes1, child_offsets, thresh1, centroids2,
                  sizes2, offsets2, thresh2, K_fixed, V_fixed, K_user, V_user, out, lse, keep_mask2, n_keys, ws, stream)


def sq_probe_stream_read(buf: torch.Tensor, sink: torch.Tensor, workgroups: int, nbytes: Optional[int] = None,
                         stream=None):
    n = buf.numel() * buf.element_size() if nbytes is None else int(nbytes)
    _check(lib().sq_probe_stream_read(_ptr(buf), n, _ptr(sink), int(workgroups), _stream(stream)))


def sq_profile_begin(max_launches: int):
    _check(lib().sq_profile_begin(int(max_launches)))


def sq_profile_end():
    """-> (launches measured, avg_us, min_us, max_us) of the split-KV partial kernel."""
    a, mn, mx = C.c_float(), C.c_float(), C.c_float()
    n = lib().sq_profile_end(C.byref(a), C.byref(mn), C.byref(mx))
    if n < 0:
        _check(n)
    return n, a.value, mn.value, mx.value


# ------------------------------------------------------------------------------------------------
# Device-resident problem: uploads a host workload once and allocates outputs.  Plumbing only.
# ------------------------------------------------------------------------------------------------
@dataclass
class DeviceProblem:
    shape: SqShape
    t: dict            # name -> device tensor

    def __getattr__(self, k):
        try:
            return self.__dict__["t"][k]
        except KeyError:
            raise AttributeError(k)


def upload(w, device="cuda:0", thresh=None) -> DeviceProblem:
    """Copy a `workload.Workload` to the device and allocate the output tensors of the one-level path.

    Masks are held as int32 tensors (torch has no uint32 arithmetic); the bits are the library's u32.
    """
    dev = torch.device(device)
    tt = lambda a: torch.from_numpy(a).to(dev)
    shape = make_shape(w.B, w.H, w.L, w.C, w.Lq, w.U, w.sm_scale, w.causal_user, w.d)
    R = (w.B, w.H, w.Lq)
    W = (w.C + 31) // 32
    th = thresh if thresh is not None else w.thresh
    t = dict(
        q=tt(w.q), centroids=tt(w.centroids), sizes=tt(w.sizes), offsets=tt(w.offsets),
        K_fixed=tt(w.K_fixed), V_fixed=tt(w.V_fixed), K_user=tt(w.K_user), V_user=tt(w.V_user),
        logits=torch.empty(*R, w.C, dtype=F32, device=dev), row_max=torch.empty(R, dtype=F32, device=dev),
        denom=torch.empty(R, dtype=F32, device=dev),
        keep_mask=torch.zeros(*R, W, dtype=I32, device=dev),
        n_ranges=torch.zeros(R, dtype=I32, device=dev), n_keys=torch.zeros(R, dtype=I32, device=dev),
        out=torch.zeros(*R, w.d, dtype=F16, device=dev), lse=torch.zeros(R, dtype=F32, device=dev),
    )
    if th is not None:
        t["thresh"] = tt(th)
    if w.Lq == 1:
        t["ranges"] = torch.zeros(*R, w.C, 2, dtype=I32, device=dev)
    if w.C1:
        t.update(centroids1=tt(w.centroids1), sizes1=tt(w.sizes1), child_offsets=tt(w.child_offsets),
                 keep_mask1=torch.zeros(w.B, w.H, (w.C1 + 31) // 32, dtype=I32, device=dev))
        if w.thresh1 is not None:
            t.update(thresh1=tt(w.thresh1), thresh2=tt(w.thresh2))
    return DeviceProblem(shape, t)
