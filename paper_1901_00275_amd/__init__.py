"""Python binding of libvlq (VLQ-ADC index for MI355X, HIP/gfx950).

Argument marshalling only: every function has the name and the argument order
of its C entry point in ``include/vlq.h`` and hands device pointers of torch
tensors to it; all computation happens in the HIP kernels of the library.
torch is used for device memory and streams.  There is no CPU fallback: a
missing library raises at the first call.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libvlq.so")

VLQ_OK, VLQ_EINVAL, VLQ_ENOMEM, VLQ_EHIP = 0, -1, -2, -3
STAGES = ("coarse", "select_cells", "subregions", "scan", "merge")
(VLQ_OPT_COARSE_FP32, VLQ_OPT_NEIGHBOURS_PER_QUERY, VLQ_OPT_SCAN_PACKED, VLQ_OPT_SCAN_GENERIC,
 VLQ_OPT_ENCODE_WAVE, VLQ_OPT_PIPELINE_PARTS, VLQ_OPT_SMALL_BATCH, VLQ_OPT_COARSE_SPLIT) = range(8)


class VlqError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"libvlq error {code}: {msg}")
        self.code = code


class vlq_params_t(C.Structure):
    _fields_ = [("d", C.c_int32), ("nlist", C.c_int32), ("n_edges", C.c_int32), ("m", C.c_int32),
                ("lambda_lo", C.c_float), ("lambda_hi", C.c_float)]


_lib = None


def lib():
    """The loaded shared library (built in-tree by ``build.py``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: run `python -m paper_1901_00275_amd.build` "
                                    "(or __graft_entry__.build()) first; there is no fallback path")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
        sig = {
            "vlq_build_index": [C.POINTER(vlq_params_t), vp, vp, vp, i64, vp, vp, C.POINTER(vp)],
            "vlq_encode": [vp, vp, i64, vp, vp, vp, vp, vp],
            "vlq_line_residuals": [vp, vp, i64, vp, vp],
            "vlq_kmeans": [vp, i64, i32, i32, i32, vp, vp, vp, vp],
            "vlq_index_add": [vp, vp, i64, vp, vp],
            "vlq_index_add_encoded": [vp, vp, vp, vp, vp, vp, i64, vp],
            "vlq_index_reserve": [vp, i64],
            "vlq_index_finalize": [vp, vp],
            "vlq_index_is_finalized": [vp],
            "vlq_index_params": [vp, C.POINTER(vlq_params_t)],
            "vlq_index_set_option": [vp, C.c_int, C.c_int],
            "vlq_index_set_query_lambda_range": [vp, C.c_float, C.c_float],
            "vlq_search": [vp, vp, i32, i32, i32, i32, vp, vp, vp],
            "vlq_search_noalloc": [vp, vp, i32, i32, i32, i32, vp, vp, vp],
            "vlq_search_debug": [vp, vp, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp],
            "vlq_index_get_graph": [vp, vp, vp, vp],
            "vlq_index_get_lists": [vp, vp, vp, vp, vp, vp],
            "vlq_profile_enable": [vp, C.c_int],
            "vlq_profile_read": [vp, C.POINTER(C.c_float), C.POINTER(i32)],
            "vlq_version": [],
        }
        for name, args in sig.items():
            fn = getattr(L, name)
            fn.argtypes = args
            fn.restype = C.c_int
        L.vlq_index_free.argtypes = [vp]
        L.vlq_index_free.restype = None
        L.vlq_index_ntotal.argtypes = [vp]
        L.vlq_index_ntotal.restype = i64
        L.vlq_last_error.argtypes = []
        L.vlq_last_error.restype = C.c_char_p
        _lib = L
    return _lib


def _chk(rc):
    if rc != 0:
        raise VlqError(rc, lib().vlq_last_error().decode())


def _ptr(t, dtype=None):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("tensors passed to libvlq must be contiguous device tensors")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"expected {dtype}, got {t.dtype}")
    return C.c_void_p(t.data_ptr())


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def vlq_version() -> int:
    return lib().vlq_version()


def vlq_last_error() -> str:
    return lib().vlq_last_error().decode()


def vlq_build_index(params: vlq_params_t, d_centroids, d_pq, d_base=None, N=0, d_ids=None, stream=None):
    """Returns the opaque index handle (free it with vlq_index_free)."""
    out = C.c_void_p()
    _chk(lib().vlq_build_index(C.byref(params), _ptr(d_centroids, torch.float32), _ptr(d_pq, torch.float32),
                               _ptr(d_base, torch.float32), int(N), _ptr(d_ids, torch.int32), _stream(stream),
                               C.byref(out)))
    return out


def vlq_index_free(idx):
    lib().vlq_index_free(idx)


def vlq_encode(idx, d_x, nb, d_cell, d_edge, d_lambda, d_codes, stream=None):
    _chk(lib().vlq_encode(idx, _ptr(d_x, torch.float32), int(nb), _ptr(d_cell, torch.int32), _ptr(d_edge, torch.int32),
                          _ptr(d_lambda, torch.uint8), _ptr(d_codes, torch.uint8), _stream(stream)))


def vlq_line_residuals(idx, d_x, nb, d_res, stream=None):
    _chk(lib().vlq_line_residuals(idx, _ptr(d_x, torch.float32), int(nb), _ptr(d_res, torch.float32), _stream(stream)))


def vlq_kmeans(d_x, nt, d, k, iters, d_centroids, d_assign=None, d_counts=None, stream=None):
    _chk(lib().vlq_kmeans(_ptr(d_x, torch.float32), int(nt), int(d), int(k), int(iters), _ptr(d_centroids, torch.float32),
                          _ptr(d_assign, torch.int32), _ptr(d_counts, torch.int32), _stream(stream)))


def vlq_index_add(idx, d_x, nb, d_ids=None, stream=None):
    _chk(lib().vlq_index_add(idx, _ptr(d_x, torch.float32), int(nb), _ptr(d_ids, torch.int32), _stream(stream)))


def vlq_index_add_encoded(idx, d_cell, d_edge, d_lambda, d_codes, d_ids, nb, stream=None):
    _chk(lib().vlq_index_add_encoded(idx, _ptr(d_cell, torch.int32), _ptr(d_edge, torch.int32),
                                     _ptr(d_lambda, torch.uint8), _ptr(d_codes, torch.uint8),
                                     _ptr(d_ids, torch.int32), int(nb), _stream(stream)))


def vlq_index_reserve(idx, total):
    _chk(lib().vlq_index_reserve(idx, int(total)))


def vlq_index_finalize(idx, stream=None):
    _chk(lib().vlq_index_finalize(idx, _stream(stream)))


def vlq_index_ntotal(idx) -> int:
    return int(lib().vlq_index_ntotal(idx))


def vlq_index_is_finalized(idx) -> bool:
    return bool(lib().vlq_index_is_finalized(idx))


def vlq_index_params(idx) -> vlq_params_t:
    p = vlq_params_t()
    _chk(lib().vlq_index_params(idx, C.byref(p)))
    return p


def vlq_index_set_option(idx, option, value):
    _chk(lib().vlq_index_set_option(idx, int(option), int(value)))


def vlq_index_set_query_lambda_range(idx, lo, hi):
    _chk(lib().vlq_index_set_query_lambda_range(idx, float(lo), float(hi)))


def vlq_search(idx, d_q, nq, w1, w2, K, d_out_dist, d_out_ids, stream=None):
    _chk(lib().vlq_search(idx, _ptr(d_q, torch.float32), int(nq), int(w1), int(w2), int(K),
                          _ptr(d_out_dist, torch.float32), _ptr(d_out_ids, torch.int32), _stream(stream)))


def vlq_search_noalloc(idx, d_q, nq, w1, w2, K, d_out_dist, d_out_ids, stream=None):
    _chk(lib().vlq_search_noalloc(idx, _ptr(d_q, torch.float32), int(nq), int(w1), int(w2), int(K),
                                  _ptr(d_out_dist, torch.float32), _ptr(d_out_ids, torch.int32), _stream(stream)))


def vlq_search_debug(idx, d_q, nq, w1, w2, K, d_out_dist, d_out_ids, d_cells=None, d_cell_dist=None, d_sub=None,
                     d_sub_score=None, stream=None):
    _chk(lib().vlq_search_debug(idx, _ptr(d_q, torch.float32), int(nq), int(w1), int(w2), int(K),
                                _ptr(d_out_dist, torch.float32), _ptr(d_out_ids, torch.int32),
                                _ptr(d_cells, torch.int32), _ptr(d_cell_dist, torch.float32),
                                _ptr(d_sub, torch.int32), _ptr(d_sub_score, torch.float32), _stream(stream)))


def vlq_index_get_graph(idx, d_S, d_E, stream=None):
    _chk(lib().vlq_index_get_graph(idx, _ptr(d_S, torch.int32), _ptr(d_E, torch.float32), _stream(stream)))


def vlq_index_get_lists(idx, d_off, d_ids, d_codes, d_lambda, stream=None):
    _chk(lib().vlq_index_get_lists(idx, _ptr(d_off, torch.int64), _ptr(d_ids, torch.int32), _ptr(d_codes, torch.uint8),
                                   _ptr(d_lambda, torch.uint8), _stream(stream)))


def vlq_profile_enable(idx, enable: bool):
    _chk(lib().vlq_profile_enable(idx, int(bool(enable))))


def vlq_profile_read(idx):
    """{stage: (milliseconds, launches)} since the last read."""
    ms = (C.c_float * len(STAGES))()
    ln = (C.c_int32 * len(STAGES))()
    _chk(lib().vlq_profile_read(idx, ms, ln))
    return {s: (float(ms[i]), int(ln[i])) for i, s in enumerate(STAGES)}
