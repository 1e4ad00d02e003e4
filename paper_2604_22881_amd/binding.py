"""ctypes binding of libmtserve_hip.so: the same entry points as include/mtserve.h.

Argument marshalling only - every step of the path runs in the HIP kernels.  PyTorch is
used for device memory and streams.  There is no fallback: if the shared library has not
been built, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(PKG_DIR, "libmtserve_hip.so")

MTS_OK, MTS_ERR_INVALID_ARG, MTS_ERR_UNSUPPORTED, MTS_ERR_SHAPE, MTS_ERR_WORKSPACE, MTS_ERR_HIP = 0, -1, -2, -3, -4, -5
MTS_ERR_BUSY = -6
MTS_F32, MTS_BF16 = 0, 1

EXPORTS = (
    "mts_page_bytes", "mts_pages_for", "mts_elem_offset", "mts_kv_unpack", "mts_kv_pack",
    "mts_kv_unpack_layers", "mts_kv_pack_layers", "mts_kv_append_layers",
    "mts_kv_append", "mts_attn_workspace_bytes", "mts_attn_set_tuning", "mts_attn_incremental", "mts_attn_incremental_noalloc", "mts_attn_pointwise",
    "mts_attn_unappended_appends", "mts_attn_incremental_unappended", "mts_attn_pointwise_unappended",
    "mts_attn_incremental_staged",
    "mts_stage_h2d_async", "mts_stage_d2h_async", "mts_diag_stream_read", "mts_last_error", "mts_version",
    "mts_xfer_create", "mts_xfer_destroy", "mts_xfer_onload_submit", "mts_xfer_onload_wait_layer",
    "mts_xfer_offload_submit", "mts_xfer_offload_pending_tokens", "mts_xfer_drain",
    "mts_cm_create", "mts_cm_destroy", "mts_cm_import_history", "mts_cm_cached_length", "mts_cm_prepare_batch", "mts_cm_commit_batch", "mts_cm_abort_batch",
    "mts_cm_offload_due", "mts_cm_offload_done", "mts_cm_set_locked", "mts_cm_take_evicted", "mts_cm_get_stats",
)


class MtsError(RuntimeError):
    def __init__(self, code, text):
        super().__init__(f"mtserve error {code}: {text}")
        self.code = code


class CacheDesc(C.Structure):
    _fields_ = [("pool", C.c_void_p), ("layer_stride_bytes", C.c_int64), ("dtype", C.c_int32),
                ("num_layers", C.c_int32), ("num_pages", C.c_int32), ("page_size", C.c_int32),
                ("num_heads", C.c_int32), ("head_dim", C.c_int32)]


class BatchMeta(C.Structure):
    _fields_ = [("batch", C.c_int32), ("page_indptr", C.c_void_p), ("page_indices", C.c_void_p),
                ("prefix_lens", C.c_void_p), ("new_indptr", C.c_void_p), ("total_new", C.c_int32),
                ("max_new", C.c_int32), ("max_total_len", C.c_int32), ("total_pages", C.c_int32)]


class AttnTuning(C.Structure):
    _fields_ = [("min_tiles", C.c_int32), ("max_waves", C.c_int32), ("pair_cost", C.c_int32), ("kernel", C.c_int32)]


MTS_ATTN_KERNEL_AUTO, MTS_ATTN_KERNEL_STREAMING, MTS_ATTN_KERNEL_PREFILL, MTS_ATTN_KERNEL_PLAIN = 0, 1, 2, 3


class XferConfig(C.Structure):
    _fields_ = [("pinned_bytes", C.c_int64), ("offload_arena_bytes", C.c_int64),
                ("offload_quota_tokens", C.c_int64), ("num_layers", C.c_int32), ("copy_threads", C.c_int32)]


class XferRuns(C.Structure):
    _fields_ = [("num_segs", C.c_int32), ("seg_user", C.c_void_p), ("seg_pos", C.c_void_p),
                ("seg_tok_indptr", C.c_void_p), ("max_seg_tokens", C.c_int32),
                ("host_tok_indptr", C.c_void_p), ("host_runs", C.c_void_p)]


class CmStats(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("gpu_hits", "host_hits", "cold_requests", "evictions", "tokens_dropped",
                                         "free_pages", "users_tracked", "users_on_gpu")]


_lib = None


def lib():
    """The loaded shared library (loaded on first use)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2604_22881_amd.build` "
            "(there is no fallback path)")
    L = C.CDLL(LIB_PATH)
    P, I32, I64, F32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
    DESC, META = C.POINTER(CacheDesc), C.POINTER(BatchMeta)
    sig = {
        "mts_page_bytes": (I64, [DESC]),
        "mts_pages_for": (I32, [I32, I32]),
        "mts_elem_offset": (I64, [DESC, I32, I32, I32, I32]),
        "mts_kv_unpack": (I32, [DESC, I32, P, I32, P, P, P, I32, META, P]),
        "mts_kv_pack": (I32, [DESC, I32, P, I32, P, P, P, I32, META, P]),
        "mts_kv_unpack_layers": (I32, [DESC, I32, I32, P, I64, I32, P, P, P, I32, META, P]),
        "mts_kv_pack_layers": (I32, [DESC, I32, I32, P, I64, I32, P, P, P, I32, META, P]),
        "mts_kv_append": (I32, [DESC, I32, P, P, META, P]),
        "mts_kv_append_layers": (I32, [DESC, I32, I32, P, P, I64, META, P]),
        "mts_attn_workspace_bytes": (I64, [DESC, META]),
        "mts_attn_set_tuning": (I32, [C.POINTER(AttnTuning)]),
        "mts_attn_incremental": (I32, [DESC, I32, P, P, META, F32, P, I64, P]),
        "mts_attn_incremental_noalloc": (I32, [DESC, I32, P, P, META, F32, P]),
        "mts_attn_pointwise": (I32, [DESC, I32, P, P, META, F32, F32, P, I64, P]),
        "mts_attn_unappended_appends": (I32, [DESC, META]),
        "mts_attn_incremental_unappended": (I32, [DESC, I32, P, P, P, P, META, F32, P, I64, P]),
        "mts_attn_pointwise_unappended": (I32, [DESC, I32, P, P, P, P, META, F32, F32, P, I64, P]),
        "mts_attn_incremental_staged": (I32, [DESC, I32, P, P, P, P, P, P, I32, P, META, F32, P, I64, P]),
        "mts_stage_h2d_async": (I32, [P, P, I64, P]),
        "mts_stage_d2h_async": (I32, [P, P, I64, P]),
        "mts_diag_stream_read": (I32, [P, I64, P, P]),
        "mts_xfer_create": (I32, [C.POINTER(XferConfig), C.POINTER(P)]),
        "mts_xfer_destroy": (I32, [P]),
        "mts_xfer_onload_submit": (I32, [P, DESC, META, C.POINTER(XferRuns), P, I64]),
        "mts_xfer_onload_wait_layer": (I32, [P, I32, P]),
        "mts_xfer_offload_submit": (I32, [P, DESC, META, C.POINTER(XferRuns), P]),
        "mts_xfer_offload_pending_tokens": (I64, [P]),
        "mts_xfer_drain": (I32, [P]),
        "mts_cm_create": (I32, [I32, I32, I32, C.POINTER(P)]),
        "mts_cm_destroy": (I32, [P]),
        "mts_cm_cached_length": (I32, [P, I64]),
        "mts_cm_import_history": (I32, [P, I64, I32]),
        "mts_cm_prepare_batch": (I32, [P, P, P, I32, P, P, P, P, I64]),
        "mts_cm_commit_batch": (I32, [P]),
        "mts_cm_abort_batch": (I32, [P]),
        "mts_cm_offload_due": (I32, [P, P, P, P, I32]),
        "mts_cm_offload_done": (I32, [P, I64, I32]),
        "mts_cm_set_locked": (I32, [P, I64, I32]),
        "mts_cm_take_evicted": (I64, [P, P, I64]),
        "mts_cm_get_stats": (I32, [P, C.POINTER(CmStats)]),
        "mts_last_error": (C.c_char_p, []),
        "mts_version": (I32, []),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype, fn.argtypes = res, args
    _lib = L
    return L


def _check(code):
    if code < 0:
        raise MtsError(int(code), lib().mts_last_error().decode())
    return code


def _ptr(x):
    """Address of a torch tensor / numpy array / int / None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if isinstance(x, np.ndarray):
        return x.ctypes.data
    return x.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


# ---- host-only helpers ------------------------------------------------------------------
def mts_version():
    return lib().mts_version()


def mts_last_error():
    return lib().mts_last_error().decode()


def mts_page_bytes(desc: CacheDesc):
    return _check(lib().mts_page_bytes(C.byref(desc)))


def mts_pages_for(length, page_size):
    return _check(lib().mts_pages_for(length, page_size))


def mts_elem_offset(desc: CacheDesc, kv, head, slot, dim):
    return _check(lib().mts_elem_offset(C.byref(desc), kv, head, slot, dim))


def mts_attn_workspace_bytes(desc: CacheDesc, meta: BatchMeta):
    return _check(lib().mts_attn_workspace_bytes(C.byref(desc), C.byref(meta)))


def mts_attn_set_tuning(min_tiles=0, max_waves=0, pair_cost=0, kernel=0):
    """Process-wide override of the attention launch plan; all zeros (the default) resets it."""
    t = AttnTuning(int(min_tiles), int(max_waves), int(pair_cost), int(kernel))
    return _check(lib().mts_attn_set_tuning(C.byref(t)))


# ---- device entry points ----------------------------------------------------------------

def mts_kv_unpack(desc, layer, staging, num_segs, seg_user, seg_pos, seg_tok_indptr, max_seg_tokens,
                  meta, stream=None):
    return _check(lib().mts_kv_unpack(C.byref(desc), layer, _ptr(staging), num_segs, _ptr(seg_user),
                                      _ptr(seg_pos), _ptr(seg_tok_indptr), max_seg_tokens,
                                      C.byref(meta), _stream(stream)))


def mts_kv_pack(desc, layer, staging_out, num_segs, seg_user, seg_pos, seg_tok_indptr, max_seg_tokens,
                meta, stream=None):
    return _check(lib().mts_kv_pack(C.byref(desc), layer, _ptr(staging_out), num_segs, _ptr(seg_user),
                                    _ptr(seg_pos), _ptr(seg_tok_indptr), max_seg_tokens,
                                    C.byref(meta), _stream(stream)))


def mts_kv_unpack_layers(desc, layer_begin, layer_count, staging, staging_layer_stride_bytes, num_segs,
                         seg_user, seg_pos, seg_tok_indptr, max_seg_tokens, meta, stream=None):
    return _check(lib().mts_kv_unpack_layers(C.byref(desc), layer_begin, layer_count, _ptr(staging),
                                             staging_layer_stride_bytes, num_segs, _ptr(seg_user),
                                             _ptr(seg_pos), _ptr(seg_tok_indptr), max_seg_tokens,
                                             C.byref(meta), _stream(stream)))


def mts_kv_pack_layers(desc, layer_begin, layer_count, staging_out, staging_layer_stride_bytes, num_segs,
                       seg_user, seg_pos, seg_tok_indptr, max_seg_tokens, meta, stream=None):
    return _check(lib().mts_kv_pack_layers(C.byref(desc), layer_begin, layer_count, _ptr(staging_out),
                                           staging_layer_stride_bytes, num_segs, _ptr(seg_user),
                                           _ptr(seg_pos), _ptr(seg_tok_indptr), max_seg_tokens,
                                           C.byref(meta), _stream(stream)))


def mts_kv_append(desc, layer, k_new, v_new, meta, stream=None):
    return _check(lib().mts_kv_append(C.byref(desc), layer, _ptr(k_new), _ptr(v_new), C.byref(meta),
                                      _stream(stream)))


def mts_kv_append_layers(desc, layer_begin, layer_count, k_new, v_new, rows_layer_stride_bytes, meta, stream=None):
    return _check(lib().mts_kv_append_layers(C.byref(desc), layer_begin, layer_count, _ptr(k_new), _ptr(v_new),
                                             int(rows_layer_stride_bytes), C.byref(meta), _stream(stream)))


def mts_attn_incremental(desc, layer, q, out, meta, sm_scale=0.0, workspace=None, workspace_bytes=0,
                         stream=None):
    return _check(lib().mts_attn_incremental(C.byref(desc), layer, _ptr(q), _ptr(out), C.byref(meta),
                                             float(sm_scale), _ptr(workspace), int(workspace_bytes),
                                             _stream(stream)))


MTS_NOALLOC_SCRATCH_BYTES = 40 << 20


def mts_attn_incremental_noalloc(desc, layer, q, out, meta, sm_scale=0.0, stream=None):
    return _check(lib().mts_attn_incremental_noalloc(C.byref(desc), layer, _ptr(q), _ptr(out), C.byref(meta),
                                                     float(sm_scale), _stream(stream)))


def mts_attn_pointwise(desc, layer, q, out, meta, inv_norm, sm_scale=0.0, workspace=None, workspace_bytes=0,
                       stream=None):
    return _check(lib().mts_attn_pointwise(C.byref(desc), layer, _ptr(q), _ptr(out), C.byref(meta),
                                           float(sm_scale), float(inv_norm), _ptr(workspace),
                                           int(workspace_bytes), _stream(stream)))


def mts_attn_unappended_appends(desc: CacheDesc, meta: BatchMeta):
    return bool(_check(lib().mts_attn_unappended_appends(C.byref(desc), C.byref(meta))))


def mts_attn_incremental_unappended(desc, layer, q, k_new, v_new, out, meta, sm_scale=0.0, workspace=None,
                                    workspace_bytes=0, stream=None):
    return _check(lib().mts_attn_incremental_unappended(C.byref(desc), layer, _ptr(q), _ptr(k_new), _ptr(v_new),
                                                        _ptr(out), C.byref(meta), float(sm_scale), _ptr(workspace),
                                                        int(workspace_bytes), _stream(stream)))


def mts_attn_pointwise_unappended(desc, layer, q, k_new, v_new, out, meta, inv_norm, sm_scale=0.0, workspace=None,
                                  workspace_bytes=0, stream=None):
    return _check(lib().mts_attn_pointwise_unappended(C.byref(desc), layer, _ptr(q), _ptr(k_new), _ptr(v_new),
                                                      _ptr(out), C.byref(meta), float(sm_scale), float(inv_norm),
                                                      _ptr(workspace), int(workspace_bytes), _stream(stream)))


def mts_attn_incremental_staged(desc, layer, q, k_new, v_new, staged_rows, staged_first_run, staged_run_tok,
                                chunk_tokens, out, meta, sm_scale=0.0, workspace=None, workspace_bytes=0, stream=None):
    return _check(lib().mts_attn_incremental_staged(C.byref(desc), layer, _ptr(q), _ptr(k_new), _ptr(v_new),
                                                    _ptr(staged_rows), _ptr(staged_first_run), _ptr(staged_run_tok),
                                                    int(chunk_tokens), _ptr(out), C.byref(meta), float(sm_scale),
                                                    _ptr(workspace), int(workspace_bytes), _stream(stream)))


# ---- transfer pipeline --------------------------------------------------------------------
def mts_xfer_create(pinned_bytes, num_layers, offload_arena_bytes=0, offload_quota_tokens=0, copy_threads=4):
    """Returns the opaque handle (an int)."""
    cfg = XferConfig(int(pinned_bytes), int(offload_arena_bytes), int(offload_quota_tokens), int(num_layers),
                     int(copy_threads))
    handle = C.c_void_p()
    _check(lib().mts_xfer_create(C.byref(cfg), C.byref(handle)))
    return handle.value


def mts_xfer_destroy(handle):
    return _check(lib().mts_xfer_destroy(handle))


def mts_xfer_onload_submit(handle, desc, meta, runs: XferRuns, staging, staging_layer_stride_bytes):
    return _check(lib().mts_xfer_onload_submit(handle, C.byref(desc), C.byref(meta), C.byref(runs), _ptr(staging),
                                               int(staging_layer_stride_bytes)))


def mts_xfer_onload_wait_layer(handle, layer, stream=None):
    return _check(lib().mts_xfer_onload_wait_layer(handle, int(layer), _stream(stream)))


def mts_xfer_offload_submit(handle, desc, meta, runs: XferRuns, after_stream=None):
    return _check(lib().mts_xfer_offload_submit(handle, C.byref(desc), C.byref(meta), C.byref(runs),
                                                _stream(after_stream)))


def mts_xfer_offload_pending_tokens(handle):
    return _check(lib().mts_xfer_offload_pending_tokens(handle))


def mts_xfer_drain(handle):
    return _check(lib().mts_xfer_drain(handle))


# ---- cache manager (host only) ----------------------------------------------------------------
class CacheManager:
    """Thin holder of an mts_cm handle: numpy arrays in, numpy arrays out; every decision is
    taken by the library."""

    def __init__(self, num_pages, page_size, host_chunk_tokens=1024):
        self._h = None
        h = C.c_void_p()
        _check(lib().mts_cm_create(int(num_pages), int(page_size), int(host_chunk_tokens), C.byref(h)))
        self._h = h.value
        self.num_pages, self.page_size = int(num_pages), int(page_size)

    def close(self):
        if self._h:
            lib().mts_cm_destroy(self._h)
            self._h = None

    __del__ = close

    def import_history(self, user, total_len):
        return _check(lib().mts_cm_import_history(self._h, int(user), int(total_len)))

    def cached_length(self, user):
        return _check(lib().mts_cm_cached_length(self._h, int(user)))

    def prepare_batch(self, users, new_tokens):
        """-> (prefix_lens, onload_lens, page_indptr, page_indices), host int32 arrays."""
        users = np.ascontiguousarray(users, dtype=np.int64)
        new_tokens = np.ascontiguousarray(new_tokens, dtype=np.int32)
        B = len(users)
        prefix = np.zeros(max(B, 1), np.int32); onload = np.zeros(max(B, 1), np.int32)
        indptr = np.zeros(B + 1, np.int32)
        cap = self.num_pages
        indices = np.zeros(max(cap, 1), np.int32)
        _check(lib().mts_cm_prepare_batch(self._h, users.ctypes.data, new_tokens.ctypes.data, B, prefix.ctypes.data,
                                          onload.ctypes.data, indptr.ctypes.data, indices.ctypes.data, cap))
        return prefix[:B], onload[:B], indptr, indices[:indptr[B]].copy()

    def commit_batch(self):
        return _check(lib().mts_cm_commit_batch(self._h))

    def abort_batch(self):
        return _check(lib().mts_cm_abort_batch(self._h))

    def offload_due(self, capacity=1024):
        u = np.zeros(capacity, np.int64); p = np.zeros(capacity, np.int32); c = np.zeros(capacity, np.int32)
        n = _check(lib().mts_cm_offload_due(self._h, u.ctypes.data, p.ctypes.data, c.ctypes.data, capacity))
        return u[:n].copy(), p[:n].copy(), c[:n].copy()

    def offload_done(self, user, persisted_len):
        return _check(lib().mts_cm_offload_done(self._h, int(user), int(persisted_len)))

    def set_locked(self, user, locked):
        return _check(lib().mts_cm_set_locked(self._h, int(user), int(bool(locked))))

    def take_evicted(self, capacity=1 << 16):
        u = np.zeros(capacity, np.int64)
        n = _check(lib().mts_cm_take_evicted(self._h, u.ctypes.data, capacity))
        return u[:n].copy()

    def stats(self):
        st = CmStats()
        _check(lib().mts_cm_get_stats(self._h, C.byref(st)))
        return {n: int(getattr(st, n)) for n, _ in CmStats._fields_}


def mts_stage_h2d_async(device_dst, host_src, nbytes, stream=None):
    return _check(lib().mts_stage_h2d_async(_ptr(device_dst), _ptr(host_src), int(nbytes), _stream(stream)))


def mts_stage_d2h_async(host_dst, device_src, nbytes, stream=None):
    return _check(lib().mts_stage_d2h_async(_ptr(host_dst), _ptr(device_src), int(nbytes), _stream(stream)))


def mts_diag_stream_read(src, nbytes, sink, stream=None):
    return _check(lib().mts_diag_stream_read(_ptr(src), int(nbytes), _ptr(sink), _stream(stream)))
