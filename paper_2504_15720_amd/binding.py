"""ctypes binding of libukv.so: same names as include/ukv.h, argument marshalling only.

Device memory comes from the caller (torch tensors give `data_ptr()`); streams are raw
hipStream_t handles (`torch.cuda.current_stream().cuda_stream`).  There is no fallback:
if the library has not been built, importing a function raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# UKV_LIB selects another build of the same library (development aid); default is the in-tree build.
LIB_PATH = os.environ.get("UKV_LIB") or os.path.join(_HERE, "libukv.so")

UKV_OK, UKV_EINVAL, UKV_ENOMEM, UKV_ENOSPC, UKV_EHIP = 0, -1, -2, -3, -4
UKV_MAX_SERVICES = 16
UKV_PARAM_MAX_SPANS, UKV_PARAM_MIN_SPAN_BYTES, UKV_PARAM_BLOCK_THREADS = 1, 2, 3
UKV_PARAM_HEADS_PER_SLICE, UKV_PARAM_PROFILE, UKV_PARAM_FUSED_MERGE = 4, 5, 6
UKV_PARAM_SLOTS, UKV_PARAM_TAPER, UKV_PARAM_GQA_COST_PCT, UKV_PARAM_PREFILL_XCD = 7, 8, 9, 10
UKV_PARAM_REPLAN_EVERY, UKV_PARAM_MERGE_ACQ_REL, UKV_PARAM_VALIDATE, UKV_PARAM_PREFILL_WEIGHTS = 11, 12, 13, 14
UKV_PARAM_PREFILL_FORM_USED, UKV_PARAM_PREFILL_PARTIALS_USED = 15, 16

EXPORTS = [
    "ukv_pool_create", "ukv_pool_destroy", "ukv_pool_info", "ukv_pages_for_tokens", "ukv_pages_alloc",
    "ukv_pages_free", "ukv_append", "ukv_decode_workspace_bytes", "ukv_decode_attention", "ukv_decode_step",
    "ukv_plan_create", "ukv_plan_step", "ukv_plan_lengths", "ukv_plan_destroy",
    "ukv_decode_attention_static", "ukv_prefill_workspace_bytes", "ukv_prefill_workspace_bytes_one_part",
    "ukv_prefill_attention",
    "ukv_gather",
    "ukv_scatter",
    "ukv_scatter_tokens",
    "ukv_plan_decode", "ukv_set_param", "ukv_get_param", "ukv_profile_read", "ukv_strerror", "ukv_last_error",
    "ukv_sched_create", "ukv_sched_destroy", "ukv_sched_add_request", "ukv_sched_next_batch", "ukv_sched_complete",
    "ukv_sched_pages_needed", "ukv_sched_request_info", "ukv_sched_pending",
]


class ukv_service_t(C.Structure):
    _fields_ = [("n_q_heads", C.c_uint32), ("n_kv_heads", C.c_uint32), ("head_dim", C.c_uint32),
                ("scale", C.c_float)]


class ukv_pool_desc_t(C.Structure):
    _fields_ = [("base", C.c_void_p), ("bytes", C.c_uint64), ("page_bytes", C.c_uint32),
                ("n_services", C.c_uint32), ("services", C.POINTER(ukv_service_t))]


class ukv_service_info_t(C.Structure):
    _fields_ = [("n_q_heads", C.c_uint32), ("n_kv_heads", C.c_uint32), ("head_dim", C.c_uint32),
                ("group", C.c_uint32), ("head_row_bytes", C.c_uint32), ("token_bytes", C.c_uint32),
                ("scale", C.c_float), ("heads_per_slice", C.c_uint32), ("n_slices", C.c_uint32),
                ("token_lanes", C.c_uint32), ("n_pages", C.c_uint64), ("free_pages", C.c_uint64)]


class ukv_batch_t(C.Structure):
    _fields_ = [("n_requests", C.c_uint32), ("service_id", C.c_void_p), ("ctx_len", C.c_void_p),
                ("table_off", C.c_void_p), ("page_table", C.c_void_p), ("q", C.c_void_p), ("q_off", C.c_void_p),
                ("out", C.c_void_p), ("out_off", C.c_void_p), ("new_k", C.c_void_p), ("new_v", C.c_void_p),
                ("new_off", C.c_void_p), ("n_patches", C.c_uint32), ("patch_entry", C.c_void_p),
                ("patch_page", C.c_void_p)]


class ukv_plan_io_t(C.Structure):
    _fields_ = [("page_table", C.c_void_p), ("q", C.c_void_p), ("out", C.c_void_p), ("new_k", C.c_void_p),
                ("new_v", C.c_void_p)]


class ukv_device_batch_t(C.Structure):
    _fields_ = [("n_requests", C.c_uint32), ("service_id", C.c_void_p), ("ctx_len", C.c_void_p),
                ("table_off", C.c_void_p), ("page_table", C.c_void_p), ("q", C.c_void_p), ("q_off", C.c_void_p),
                ("out", C.c_void_p), ("out_off", C.c_void_p)]


UKV_STATIC_SCRATCH_BYTES, UKV_STATIC_MAX_REQUESTS = 16 << 20, 1024


class ukv_plan_info_t(C.Structure):
    _fields_ = [("n_seqs", C.c_uint32), ("n_items", C.c_uint32), ("n_spans", C.c_uint32), ("n_reduce", C.c_uint32),
                ("partial_floats", C.c_uint64), ("plan_bytes", C.c_uint64), ("kv_bytes", C.c_uint64)]


class ukv_profile_t(C.Structure):
    _fields_ = [("n_decode", C.c_uint32), ("n_reduce", C.c_uint32), ("n_append", C.c_uint32),
                ("n_prefill", C.c_uint32),
                ("decode_ms", C.c_double), ("reduce_ms", C.c_double), ("append_ms", C.c_double),
                ("prefill_ms", C.c_double)]


class ukv_sched_service_t(C.Structure):
    _fields_ = [("mean_time", C.c_double), ("std_time", C.c_double), ("starvation_threshold", C.c_double)]


class ukv_sched_request_t(C.Structure):
    _fields_ = [("service", C.c_uint32), ("queue", C.c_uint32), ("prompt_len", C.c_uint32), ("ctx_len", C.c_uint32),
                ("doublings", C.c_uint32), ("arrival", C.c_double), ("budget", C.c_double), ("priority", C.c_double)]


UKV_SCHED_WAIT, UKV_SCHED_DECODING = 0, 1


class UkvError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(f"{what}: {ukv_strerror(code)} ({code}): {ukv_last_error()}")


_lib = None


def lib():
    """The loaded library; raises if it has not been built (no fallback path exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
        L = C.CDLL(LIB_PATH)
        vp = C.c_void_p
        L.ukv_pool_create.argtypes = [C.POINTER(ukv_pool_desc_t), C.POINTER(vp)]
        L.ukv_pool_destroy.argtypes = [vp]
        L.ukv_pool_info.argtypes = [vp, C.c_uint32, C.POINTER(ukv_service_info_t)]
        L.ukv_pages_for_tokens.argtypes = [vp, C.c_uint32, C.c_uint64]
        L.ukv_pages_for_tokens.restype = C.c_uint64
        L.ukv_pages_alloc.argtypes = [vp, C.c_uint32, vp]
        L.ukv_pages_free.argtypes = [vp, C.c_uint32, vp]
        L.ukv_append.argtypes = [vp, C.POINTER(ukv_batch_t), vp]
        L.ukv_decode_workspace_bytes.argtypes = [vp, C.c_uint32]
        L.ukv_decode_workspace_bytes.restype = C.c_size_t
        L.ukv_decode_attention.argtypes = [vp, C.POINTER(ukv_batch_t), vp, C.c_size_t, vp]
        L.ukv_decode_step.argtypes = [vp, C.POINTER(ukv_batch_t), vp, C.c_size_t, vp]
        L.ukv_plan_create.argtypes = [vp, C.POINTER(ukv_batch_t), vp, C.c_size_t, C.POINTER(vp)]
        L.ukv_plan_step.argtypes = [vp, C.POINTER(ukv_plan_io_t), C.c_int, vp, C.c_uint32, vp]
        L.ukv_plan_lengths.argtypes = [vp, vp, C.c_uint32]
        L.ukv_plan_destroy.argtypes = [vp]
        L.ukv_decode_attention_static.argtypes = [vp, C.POINTER(ukv_device_batch_t), vp]
        L.ukv_prefill_workspace_bytes.argtypes = [vp, C.c_uint32, C.c_uint64]
        L.ukv_prefill_workspace_bytes.restype = C.c_size_t
        L.ukv_prefill_workspace_bytes_one_part.argtypes = [vp, C.c_uint32, C.c_uint64, C.c_uint64]
        L.ukv_prefill_workspace_bytes_one_part.restype = C.c_size_t
        L.ukv_prefill_attention.argtypes = [vp, C.POINTER(ukv_batch_t), vp, vp, C.c_size_t, vp]
        L.ukv_gather.argtypes = [vp, C.POINTER(ukv_batch_t), vp, vp, vp, vp]
        L.ukv_scatter.argtypes = [vp, C.POINTER(ukv_batch_t), vp, vp, vp, vp]
        L.ukv_scatter_tokens.argtypes = [vp, C.POINTER(ukv_batch_t), vp, vp, vp, vp, vp]
        L.ukv_plan_decode.argtypes = [vp, C.POINTER(ukv_batch_t), C.POINTER(ukv_plan_info_t), vp, C.c_uint32]
        L.ukv_set_param.argtypes = [vp, C.c_int, C.c_int64]
        L.ukv_get_param.argtypes = [vp, C.c_int, C.POINTER(C.c_int64)]
        L.ukv_profile_read.argtypes = [vp, C.POINTER(ukv_profile_t)]
        L.ukv_sched_create.argtypes = [vp, C.POINTER(ukv_sched_service_t), C.c_uint32, C.c_uint32, C.POINTER(vp)]
        L.ukv_sched_destroy.argtypes = [vp]
        L.ukv_sched_add_request.argtypes = [vp, C.c_uint64, C.c_uint32, C.c_uint32, C.c_double]
        L.ukv_sched_next_batch.argtypes = [vp, C.c_double, C.c_uint64, vp, C.c_uint32, C.POINTER(C.c_uint32),
                                           C.POINTER(C.c_uint32), C.POINTER(C.c_uint32)]
        L.ukv_sched_complete.argtypes = [vp, vp, vp, C.c_uint32, C.c_double, C.c_double]
        L.ukv_sched_pages_needed.argtypes = [vp, C.c_uint64, C.POINTER(C.c_uint64)]
        L.ukv_sched_request_info.argtypes = [vp, C.c_uint64, C.POINTER(ukv_sched_request_t)]
        L.ukv_sched_pending.argtypes = [vp]
        L.ukv_sched_pending.restype = C.c_uint32
        L.ukv_strerror.argtypes = [C.c_int]
        L.ukv_strerror.restype = C.c_char_p
        L.ukv_last_error.restype = C.c_char_p
        _lib = L
    return _lib


def _check(rc: int, what: str) -> None:
    if rc != UKV_OK:
        raise UkvError(rc, what)


def ukv_strerror(code: int) -> str:
    return lib().ukv_strerror(code).decode()


def ukv_last_error() -> str:
    return lib().ukv_last_error().decode()


def ukv_pool_create(base_ptr: int, n_bytes: int, page_bytes: int, services: Sequence) -> int:
    """services: objects with n_q_heads, n_kv_heads, head_dim, scale.  Returns the pool handle."""
    arr = (ukv_service_t * len(services))()
    for i, s in enumerate(services):
        arr[i] = ukv_service_t(s.n_q_heads, s.n_kv_heads, s.head_dim, float(getattr(s, "scale", 0.0)))
    desc = ukv_pool_desc_t(base_ptr, n_bytes, page_bytes, len(services), arr)
    out = C.c_void_p()
    _check(lib().ukv_pool_create(C.byref(desc), C.byref(out)), "ukv_pool_create")
    return out.value


def ukv_pool_destroy(pool: int) -> None:
    _check(lib().ukv_pool_destroy(pool), "ukv_pool_destroy")


def ukv_pool_info(pool: int, service: int) -> ukv_service_info_t:
    info = ukv_service_info_t()
    _check(lib().ukv_pool_info(pool, service, C.byref(info)), "ukv_pool_info")
    return info


def ukv_pages_for_tokens(pool: int, service: int, n_tokens: int) -> int:
    return int(lib().ukv_pages_for_tokens(pool, service, n_tokens))


def ukv_pages_alloc(pool: int, n: int) -> np.ndarray:
    ids = np.empty(n, np.int32)
    _check(lib().ukv_pages_alloc(pool, n, ids.ctypes.data), "ukv_pages_alloc")
    return ids


def ukv_pages_free(pool: int, ids) -> None:
    ids = np.ascontiguousarray(ids, np.int32)
    _check(lib().ukv_pages_free(pool, ids.size, ids.ctypes.data), "ukv_pages_free")


def ukv_set_param(pool: int, key: int, value: int) -> None:
    _check(lib().ukv_set_param(pool, key, value), "ukv_set_param")


def ukv_get_param(pool: int, key: int) -> int:
    v = C.c_int64()
    _check(lib().ukv_get_param(pool, key, C.byref(v)), "ukv_get_param")
    return int(v.value)


class BatchDesc:
    """Holds the host arrays alive and the ukv_batch_t that points at them."""

    def __init__(self, service_id, ctx_len, table_off, page_table_ptr: int = 0, q_ptr: int = 0, q_off=None,
                 out_ptr: int = 0, out_off=None, new_k_ptr: int = 0, new_v_ptr: int = 0, new_off=None,
                 patch_entry=None, patch_page=None):
        n = len(service_id)
        self.service_id = np.ascontiguousarray(service_id, np.uint32)
        self.ctx_len = np.ascontiguousarray(ctx_len, np.uint32)
        self.table_off = np.ascontiguousarray(table_off, np.uint64)
        zeros = np.zeros(n, np.uint64)
        self.q_off = np.ascontiguousarray(q_off if q_off is not None else zeros, np.uint64)
        self.out_off = np.ascontiguousarray(out_off if out_off is not None else zeros, np.uint64)
        self.new_off = np.ascontiguousarray(new_off if new_off is not None else zeros, np.uint64)
        self.patch_entry = np.ascontiguousarray(patch_entry if patch_entry is not None else [], np.uint64)
        self.patch_page = np.ascontiguousarray(patch_page if patch_page is not None else [], np.int32)
        assert self.patch_entry.size == self.patch_page.size
        self.c = ukv_batch_t(n, self.service_id.ctypes.data, self.ctx_len.ctypes.data, self.table_off.ctypes.data,
                             page_table_ptr, q_ptr, self.q_off.ctypes.data, out_ptr, self.out_off.ctypes.data,
                             new_k_ptr, new_v_ptr, self.new_off.ctypes.data, self.patch_entry.size,
                             self.patch_entry.ctypes.data if self.patch_entry.size else None,
                             self.patch_page.ctypes.data if self.patch_page.size else None)


def ukv_append(pool: int, batch: BatchDesc, stream: int = 0) -> None:
    _check(lib().ukv_append(pool, C.byref(batch.c), stream), "ukv_append")


def ukv_decode_workspace_bytes(pool: int, n_requests: int) -> int:
    return int(lib().ukv_decode_workspace_bytes(pool, n_requests))


def ukv_decode_attention(pool: int, batch: BatchDesc, workspace_ptr: int, ws_bytes: int, stream: int = 0) -> None:
    _check(lib().ukv_decode_attention(pool, C.byref(batch.c), workspace_ptr, ws_bytes, stream),
           "ukv_decode_attention")


def ukv_decode_step(pool: int, batch: BatchDesc, workspace_ptr: int, ws_bytes: int, stream: int = 0) -> None:
    _check(lib().ukv_decode_step(pool, C.byref(batch.c), workspace_ptr, ws_bytes, stream), "ukv_decode_step")


def ukv_plan_create(pool: int, batch: BatchDesc, workspace_ptr: int, ws_bytes: int) -> int:
    out = C.c_void_p()
    _check(lib().ukv_plan_create(pool, C.byref(batch.c), workspace_ptr, ws_bytes, C.byref(out)), "ukv_plan_create")
    return out.value


def ukv_plan_step(plan: int, new_pages, advance: bool = True, io=None, stream: int = 0) -> None:
    """io: None, or (page_table_ptr, q_ptr, out_ptr, new_k_ptr, new_v_ptr)."""
    pages = np.ascontiguousarray(new_pages, np.int32)
    io_c = C.byref(ukv_plan_io_t(*io)) if io is not None else None
    _check(lib().ukv_plan_step(plan, io_c, 1 if advance else 0, pages.ctypes.data if pages.size else None, pages.size,
                               stream), "ukv_plan_step")


def ukv_plan_lengths(plan: int, n: int) -> np.ndarray:
    out = np.zeros(n, np.uint32)
    _check(lib().ukv_plan_lengths(plan, out.ctypes.data, n), "ukv_plan_lengths")
    return out


def ukv_plan_destroy(plan: int) -> None:
    _check(lib().ukv_plan_destroy(plan), "ukv_plan_destroy")


def ukv_decode_attention_static(pool: int, n_requests: int, service_id_ptr: int, ctx_len_ptr: int, table_off_ptr: int,
                                page_table_ptr: int, q_ptr: int, q_off_ptr: int, out_ptr: int, out_off_ptr: int,
                                stream: int = 0) -> None:
    """Every pointer is device memory (see ukv_device_batch_t)."""
    d = ukv_device_batch_t(n_requests, service_id_ptr, ctx_len_ptr, table_off_ptr, page_table_ptr, q_ptr, q_off_ptr,
                           out_ptr, out_off_ptr)
    _check(lib().ukv_decode_attention_static(pool, C.byref(d), stream), "ukv_decode_attention_static")


def ukv_prefill_workspace_bytes(pool: int, n_requests: int, total_q_rows: int) -> int:
    return int(lib().ukv_prefill_workspace_bytes(pool, n_requests, total_q_rows))


def ukv_prefill_workspace_bytes_one_part(pool: int, n_requests: int, total_q_rows: int, total_ctx_tokens: int) -> int:
    return int(lib().ukv_prefill_workspace_bytes_one_part(pool, n_requests, total_q_rows, total_ctx_tokens))


def ukv_prefill_attention(pool: int, batch: BatchDesc, q_len, workspace_ptr: int, ws_bytes: int,
                          stream: int = 0) -> None:
    q_len = np.ascontiguousarray(q_len, np.uint32)
    _check(lib().ukv_prefill_attention(pool, C.byref(batch.c), q_len.ctypes.data, workspace_ptr, ws_bytes, stream),
           "ukv_prefill_attention")


def ukv_gather(pool: int, batch: BatchDesc, k_out_ptr: int, v_out_ptr: int, kv_off, stream: int = 0) -> None:
    kv_off = np.ascontiguousarray(kv_off, np.uint64)
    _check(lib().ukv_gather(pool, C.byref(batch.c), k_out_ptr, v_out_ptr, kv_off.ctypes.data, stream), "ukv_gather")


def ukv_scatter(pool: int, batch: BatchDesc, k_in_ptr: int, v_in_ptr: int, kv_off, stream: int = 0) -> None:
    kv_off = np.ascontiguousarray(kv_off, np.uint64)
    _check(lib().ukv_scatter(pool, C.byref(batch.c), k_in_ptr, v_in_ptr, kv_off.ctypes.data, stream), "ukv_scatter")


def ukv_scatter_tokens(pool: int, batch: BatchDesc, n_new, k_in_ptr: int, v_in_ptr: int, kv_off,
                       stream: int = 0) -> None:
    n_new = np.ascontiguousarray(n_new, np.uint32)
    kv_off = np.ascontiguousarray(kv_off, np.uint64)
    _check(lib().ukv_scatter_tokens(pool, C.byref(batch.c), n_new.ctypes.data, k_in_ptr, v_in_ptr, kv_off.ctypes.data,
                                    stream), "ukv_scatter_tokens")


def ukv_plan_decode(pool: int, batch: BatchDesc, want_items: bool = True):
    """Returns (ukv_plan_info_t, items[n_items, 6] = request, head0, n_heads, t0, t1, span)."""
    info = ukv_plan_info_t()
    _check(lib().ukv_plan_decode(pool, C.byref(batch.c), C.byref(info), None, 0), "ukv_plan_decode")
    items = None
    if want_items:
        items = np.zeros((info.n_items, 6), np.uint32)
        _check(lib().ukv_plan_decode(pool, C.byref(batch.c), C.byref(info), items.ctypes.data, info.n_items),
               "ukv_plan_decode")
    return info, items


def ukv_sched_create(pool: int, profiles, max_batch: int) -> int:
    """profiles: (mean_time, std_time, starvation_threshold) per service of the pool."""
    arr = (ukv_sched_service_t * len(profiles))(*[ukv_sched_service_t(*map(float, p)) for p in profiles])
    out = C.c_void_p()
    _check(lib().ukv_sched_create(pool, arr, len(profiles), max_batch, C.byref(out)), "ukv_sched_create")
    return out.value


def ukv_sched_destroy(sched: int) -> None:
    _check(lib().ukv_sched_destroy(sched), "ukv_sched_destroy")


def ukv_sched_add_request(sched: int, rid: int, service: int, prompt_len: int, now: float) -> None:
    _check(lib().ukv_sched_add_request(sched, rid, service, prompt_len, now), "ukv_sched_add_request")


def ukv_sched_next_batch(sched: int, now: float, free_pages: int, cap: int = 4096):
    """Returns (ids, service, queue)."""
    ids = np.zeros(cap, np.uint64)
    n, svc, queue = C.c_uint32(), C.c_uint32(), C.c_uint32()
    _check(lib().ukv_sched_next_batch(sched, now, free_pages, ids.ctypes.data, cap, C.byref(n), C.byref(svc),
                                      C.byref(queue)), "ukv_sched_next_batch")
    return [int(x) for x in ids[:n.value]], int(svc.value), int(queue.value)


def ukv_sched_complete(sched: int, ids, finished, elapsed: float, now: float) -> None:
    ids = np.ascontiguousarray(ids, np.uint64)
    fin = np.ascontiguousarray(finished, np.uint8)
    _check(lib().ukv_sched_complete(sched, ids.ctypes.data, fin.ctypes.data, ids.size, elapsed, now),
           "ukv_sched_complete")


def ukv_sched_pages_needed(sched: int, rid: int) -> int:
    out = C.c_uint64()
    _check(lib().ukv_sched_pages_needed(sched, rid, C.byref(out)), "ukv_sched_pages_needed")
    return int(out.value)


def ukv_sched_request_info(sched: int, rid: int) -> ukv_sched_request_t:
    out = ukv_sched_request_t()
    _check(lib().ukv_sched_request_info(sched, rid, C.byref(out)), "ukv_sched_request_info")
    return out


def ukv_sched_pending(sched: int) -> int:
    return int(lib().ukv_sched_pending(sched))


def ukv_profile_read(pool: int) -> ukv_profile_t:
    prof = ukv_profile_t()
    _check(lib().ukv_profile_read(pool, C.byref(prof)), "ukv_profile_read")
    return prof
