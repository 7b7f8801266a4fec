"""ctypes binding of liblora_cache.so: argument marshalling only.

Every function has the name it has in include/lora_cache.h and returns what the C call
returns (a status, or a size); `check()` turns a negative status into LoraError.  Device
buffers are passed as integers (`tensor.data_ptr()`), streams as `torch.cuda.Stream.cuda_stream`.
The library is required: importing this module fails loudly when the shared object has not
been built (python -m paper_2411_17741_amd.build, or __graft_entry__.build()).
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, c_char_p, c_float, c_int, c_int32, c_int64, c_size_t, c_void_p
from typing import Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("LORA_CACHE_LIB") or os.path.join(_HERE, "liblora_cache.so")  # the variable names another build of the same library

LORA_OK, LORA_E_INVAL, LORA_E_STATE, LORA_E_NOMEM, LORA_E_HIP, LORA_E_NOTFOUND, LORA_E_FAULT = 0, -1, -2, -3, -4, -5, -6
LORA_F32, LORA_BF16 = 0, 1
LORA_SLOT_EMPTY, LORA_SLOT_FILLING, LORA_SLOT_READY = 0, 1, 2
LORA_CACHE_HOST_ONLY, LORA_CACHE_FUSED_GEMV, LORA_CACHE_SPLIT_GEMV, LORA_CACHE_DIRECT_FILL, LORA_CACHE_NO_OVERLAP = 1, 2, 4, 8, 16
LORA_MAX_RANK, LORA_TILE_TOKENS, LORA_MFMA_MIN_TOKENS, LORA_MFMA_MIN_TOKENS_MIXED = 128, 64, 16, 8


class LoraError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__(f"{what}: {lora_strerror(status)} ({status})" + (f", hip error {lora_last_hip_error()}" if status == LORA_E_HIP else ""))
        self.status = status


class lora_proj_t(ctypes.Structure):
    _fields_ = [("h_in", c_int32), ("h_out", c_int32)]


class lora_cache_config_t(ctypes.Structure):
    _fields_ = [
        ("n_proj", c_int32), ("proj", POINTER(lora_proj_t)), ("n_layers", c_int32), ("n_classes", c_int32),
        ("class_rank", POINTER(c_int32)), ("class_slots", POINTER(c_int32)), ("dtype", c_int32),
        ("max_tokens", c_int32), ("max_segments", c_int32), ("n_plans", c_int32), ("mfma_min_tokens", c_int32),
        ("flags", c_int32),
    ]


class lora_slot_info_t(ctypes.Structure):
    _fields_ = [
        ("adapter_id", c_int64), ("rank", c_int32), ("class_rank", c_int32), ("state", c_int32), ("refcount", c_int32),
        ("use_count", c_int64), ("last_used", c_int64), ("alpha", c_float), ("parts_filled", c_int32),
    ]


class lora_sched_config_t(ctypes.Structure):
    _fields_ = [("n_queues", c_int32), ("quota", POINTER(c_int64)), ("boundaries", POINTER(ctypes.c_double)),
                ("max_input", c_int32), ("max_output", c_int32), ("max_rank", c_int32), ("tokens_per_rank", c_int32),
                ("a_input", ctypes.c_double), ("b_output", ctypes.c_double)]


class lora_policy_t(ctypes.Structure):
    _fields_ = [("w_freq", ctypes.c_double), ("w_recency", ctypes.c_double), ("w_size", ctypes.c_double), ("freq_window", c_int64)]


class lora_cache_stats_t(ctypes.Structure):
    _fields_ = [(n, c_int64) for n in ("hits", "misses", "fills", "bytes_filled", "applies", "evictions")]


class lora_item_t(ctypes.Structure):
    _fields_ = [(n, c_int32) for n in ("tok_off", "n_tok", "slot", "rank", "a", "b", "c", "d")]


class lora_plan_info_t(ctypes.Structure):
    _fields_ = [(n, c_int32) for n in ("T", "mfma_min_tokens", "n_tiles", "n_tile_tokens", "n_gemv_shrink_items", "n_gemv_expand_items")]


class lora_apply_desc_t(ctypes.Structure):
    _fields_ = [("layer", c_int32), ("proj", c_int32), ("x", c_void_p), ("base_out", c_void_p)]

class lora_fill_part_t(ctypes.Structure):
    _fields_ = [("layer", c_int32), ("proj", c_int32), ("host_A", c_void_p), ("host_B", c_void_p)]


class lora_worklists_t(ctypes.Structure):
    _fields_ = [
        ("n_tok_list", c_int32), ("n_tiles", c_int32), ("n_groups", c_int32),
        ("tok_list", POINTER(c_int32)), ("tiles", POINTER(lora_item_t)), ("groups", POINTER(lora_item_t)),
    ]


LORA_UNIT_TILE, LORA_UNIT_GEMV_SHRINK, LORA_UNIT_GEMV_EXPAND, LORA_UNIT_LINEAR_ROWS, LORA_UNIT_TILE_SHRINK, LORA_UNIT_TILE_SUM = 0, 1, 2, 3, 4, 5


class lora_plan_unit_t(ctypes.Structure):
    _fields_ = [(n, c_int32) for n in ("kind", "tok_off", "n_tok", "slot", "rank", "lo", "hi", "where")] + [("alpha", c_float)]


if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `python -m paper_2411_17741_amd.build` "
        "(there is no fallback path; the HIP library is the product)"
    )
_lib = ctypes.CDLL(LIB_PATH)

_i32p = POINTER(c_int32)
_SIGS = {
    "lora_adapter_bytes": (c_size_t, [c_int32, c_int32, c_int32, c_int32]),
    "lora_cache_bytes_required": (c_size_t, [POINTER(lora_cache_config_t)]),
    "lora_cache_create": (c_int, [POINTER(lora_cache_config_t), c_void_p, c_size_t, POINTER(c_void_p)]),
    "lora_cache_destroy": (c_int, [c_void_p]),
    "lora_cache_fill_slot": (c_int, [c_void_p, c_int32, c_int64, c_int32, c_float, c_int32, c_int32, c_void_p, c_void_p, c_void_p]),
    "lora_cache_fill_slot_parts": (c_int, [c_void_p, c_int32, c_int64, c_int32, c_float, c_void_p, c_int32, c_void_p]),
    "lora_cache_release_slot": (c_int, [c_void_p, c_int32]),
    "lora_cache_slot_ref": (c_int, [c_void_p, c_int32, c_int32]),
    "lora_cache_lookup": (c_int, [c_void_p, c_int64, _i32p, _i32p]),
    "lora_cache_slot_info": (c_int, [c_void_p, c_int32, POINTER(lora_slot_info_t)]),
    "lora_cache_slot_state": (c_int, [c_void_p, c_int32, _i32p]),
    "lora_cache_find_free_slot": (c_int, [c_void_p, c_int32, _i32p]),
    "lora_cache_stats": (c_int, [c_void_p, POINTER(lora_cache_stats_t)]),
    "lora_cache_set_policy": (c_int, [c_void_p, POINTER(lora_policy_t)]),
    "lora_cache_get_policy": (c_int, [c_void_p, POINTER(lora_policy_t)]),
    "lora_cache_acquire": (c_int, [c_void_p, c_int64, c_int32, c_float, c_int32, POINTER(c_int64), c_int32, _i32p, _i32p]),
    "lora_cache_score": (c_int, [c_void_p, c_int32, POINTER(ctypes.c_double)]),
    "lora_cache_choose_victim": (c_int, [c_void_p, c_int32, POINTER(c_int64), c_int32, _i32p]),
    "lora_cache_resident_bytes": (c_int, [c_void_p, POINTER(c_size_t)]),
    "lora_cache_trim": (c_int, [c_void_p, c_size_t, POINTER(c_int64), c_int32, _i32p]),
    "lora_cache_slab": (c_int, [c_void_p, c_int32, c_int32, c_int32, POINTER(c_void_p), POINTER(c_size_t)]),
    "lora_index": (c_int, [c_int32, _i32p, _i32p, _i32p, c_int32, c_int32, POINTER(lora_worklists_t)]),
    "lora_worklists_free": (None, [POINTER(lora_worklists_t)]),
    "lora_plan_create": (c_int, [c_void_p, c_int32, _i32p, _i32p, _i32p, c_int32, c_void_p, POINTER(c_void_p)]),
    "lora_plan_destroy": (c_int, [c_void_p, c_void_p]),
    "lora_plan_info": (c_int, [c_void_p, POINTER(lora_plan_info_t)]),
    "lora_plan_dump": (c_int, [c_void_p, c_void_p, c_int32, POINTER(lora_plan_unit_t), c_int32, _i32p, _i32p, c_int32, _i32p]),
    "lora_apply_plan": (c_int, [c_void_p, c_void_p, c_int32, c_int32, c_void_p, c_void_p, c_float, c_void_p]),
    "lora_apply_plan_static": (c_int, [c_void_p, c_void_p, c_int32, c_int32, c_void_p, c_void_p, c_float, c_void_p]),
    "lora_apply_plan_multi": (c_int, [c_void_p, c_void_p, POINTER(lora_apply_desc_t), c_int32, c_float, c_void_p]),
    "lora_linear_plan": (c_int, [c_void_p, c_void_p, c_int32, c_int32, c_void_p, c_void_p, c_void_p, c_float, c_void_p, c_size_t, c_void_p]),
    "lora_linear_workspace_bytes": (c_int, [c_void_p, c_void_p, c_int32, POINTER(c_size_t)]),
    "lora_apply": (c_int, [c_void_p, c_int32, c_int32, c_void_p, c_void_p, c_int32, _i32p, _i32p, _i32p, c_int32, c_float, c_void_p]),
    "lora_cache_set_fencing": (c_int, [c_void_p, c_int32]),
    "lora_cache_set_timing": (c_int, [c_void_p, c_int32]),
    "lora_cache_read_timing": (c_int, [c_void_p, POINTER(ctypes.c_double), POINTER(c_int64)]),
    "lora_cache_check_fault": (c_int, [c_void_p, c_void_p, _i32p]),
    "lora_sched_wrs": (ctypes.c_double, [c_int32, c_int32, c_int32, c_int32, c_int32, c_int32, ctypes.c_double, ctypes.c_double]),
    "lora_sched_create": (c_int, [POINTER(lora_sched_config_t), POINTER(c_void_p)]),
    "lora_sched_destroy": (c_int, [c_void_p]),
    "lora_sched_submit": (c_int, [c_void_p, c_int64, c_int32, c_int32, c_int64, c_int32, _i32p]),
    "lora_sched_generate_batch": (c_int, [c_void_p, POINTER(c_int64), c_int32, _i32p]),
    "lora_sched_finish": (c_int, [c_void_p, c_int64]),
    "lora_sched_queue_state": (c_int, [c_void_p, c_int32, POINTER(c_int64), _i32p]),
    "lora_sched_waiting_adapters": (c_int, [c_void_p, POINTER(c_int64), c_int32, _i32p]),
    "lora_sched_fit_queues": (c_int, [POINTER(ctypes.c_double), c_int32, c_int32, _i32p, POINTER(ctypes.c_double)]),
    "lora_sched_min_quota": (c_int64, [ctypes.c_double, ctypes.c_double, ctypes.c_double, ctypes.c_double]),
    "lora_sched_assign_quotas": (c_int, [c_int64, POINTER(c_int64), POINTER(ctypes.c_double), c_int32, POINTER(c_int64)]),
    "lora_strerror": (c_char_p, [c_int]),
    "lora_last_hip_error": (c_int, []),
}
EXPORTS = tuple(_SIGS)
for _name, (_res, _args) in _SIGS.items():
    _fn = getattr(_lib, _name)  # AttributeError here = the library does not export a declared symbol
    _fn.restype = _res
    _fn.argtypes = _args


def lora_strerror(status: int) -> str:
    return _lib.lora_strerror(int(status)).decode()


def lora_last_hip_error() -> int:
    return int(_lib.lora_last_hip_error())


def check(status: int, what: str = "liblora_cache") -> int:
    if status < 0:
        raise LoraError(status, what)
    return status


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(_i32p)


def make_config(proj: Sequence[Sequence[int]], n_layers: int, class_rank: Sequence[int], class_slots: Sequence[int],
                dtype: int, max_tokens: int, max_segments: int, n_plans: int = 2, mfma_min_tokens: int = 0, flags: int = 0):
    """Returns (config struct, keep-alive tuple of the arrays it points to)."""
    pa = (lora_proj_t * len(proj))(*[lora_proj_t(int(a), int(b)) for a, b in proj])
    cr = (c_int32 * len(class_rank))(*[int(v) for v in class_rank])
    cs = (c_int32 * len(class_slots))(*[int(v) for v in class_slots])
    cfg = lora_cache_config_t(len(proj), pa, int(n_layers), len(class_rank), cr, cs, int(dtype), int(max_tokens),
                              int(max_segments), int(n_plans), int(mfma_min_tokens), int(flags))
    cfg._keep = (pa, cr, cs)
    return cfg


def lora_adapter_bytes(h_in: int, h_out: int, rank: int, dtype: int) -> int:
    return int(_lib.lora_adapter_bytes(h_in, h_out, rank, dtype))


def lora_cache_bytes_required(cfg: lora_cache_config_t) -> int:
    return int(_lib.lora_cache_bytes_required(ctypes.byref(cfg)))


def lora_cache_create(cfg: lora_cache_config_t, dev_pool: int, dev_pool_bytes: int):
    """-> (status, handle)"""
    h = c_void_p()
    rc = _lib.lora_cache_create(ctypes.byref(cfg), c_void_p(dev_pool or None), dev_pool_bytes, ctypes.byref(h))
    return rc, h


def lora_cache_destroy(cache) -> int:
    return _lib.lora_cache_destroy(cache)


def lora_cache_fill_slot(cache, slot: int, adapter_id: int, rank: int, alpha: float, layer: int, proj: int,
                         host_A: int, host_B: int, fill_stream: int = 0) -> int:
    return _lib.lora_cache_fill_slot(cache, slot, adapter_id, rank, alpha, layer, proj, c_void_p(host_A or None),
                                     c_void_p(host_B or None), c_void_p(fill_stream or None))


def make_fill_parts(entries):
    """[(layer, proj, host_A address, host_B address), ...] -> C array for lora_cache_fill_slot_parts."""
    arr = (lora_fill_part_t * len(entries))()
    for i, (layer, proj, a, b) in enumerate(entries):
        arr[i] = lora_fill_part_t(int(layer), int(proj), c_void_p(a or None), c_void_p(b or None))
    return arr


def lora_cache_fill_slot_parts(cache, slot: int, adapter_id: int, rank: int, alpha: float, parts, fill_stream: int = 0) -> int:
    return _lib.lora_cache_fill_slot_parts(cache, slot, adapter_id, rank, alpha, ctypes.cast(parts, c_void_p), len(parts),
                                           c_void_p(fill_stream or None))


def lora_cache_release_slot(cache, slot: int) -> int:
    return _lib.lora_cache_release_slot(cache, slot)


def lora_cache_slot_ref(cache, slot: int, delta: int) -> int:
    return _lib.lora_cache_slot_ref(cache, slot, delta)


def lora_cache_lookup(cache, adapter_id: int):
    """-> (status, slot, rank)"""
    s, r = c_int32(-1), c_int32(0)
    rc = _lib.lora_cache_lookup(cache, adapter_id, ctypes.byref(s), ctypes.byref(r))
    return rc, s.value, r.value


def lora_cache_slot_info(cache, slot: int):
    """-> (status, lora_slot_info_t)"""
    info = lora_slot_info_t()
    rc = _lib.lora_cache_slot_info(cache, slot, ctypes.byref(info))
    return rc, info


def lora_cache_slot_state(cache, slot: int):
    """-> (status, state)"""
    st = c_int32(-1)
    rc = _lib.lora_cache_slot_state(cache, slot, ctypes.byref(st))
    return rc, st.value


def lora_cache_find_free_slot(cache, rank: int):
    s = c_int32(-1)
    rc = _lib.lora_cache_find_free_slot(cache, rank, ctypes.byref(s))
    return rc, s.value


def lora_cache_stats(cache):
    st = lora_cache_stats_t()
    rc = _lib.lora_cache_stats(cache, ctypes.byref(st))
    return rc, st


def _ids(queued_ids):
    q = np.ascontiguousarray(np.asarray(queued_ids if queued_ids is not None else [], dtype=np.int64))
    return q, (q.ctypes.data_as(POINTER(c_int64)) if q.size else None), int(q.size)


def lora_cache_set_policy(cache, w_freq: float, w_recency: float, w_size: float, freq_window: int = 0) -> int:
    pol = lora_policy_t(w_freq, w_recency, w_size, freq_window)
    return _lib.lora_cache_set_policy(cache, ctypes.byref(pol))


def lora_cache_get_policy(cache):
    """-> (status, (w_freq, w_recency, w_size, freq_window))"""
    pol = lora_policy_t()
    rc = _lib.lora_cache_get_policy(cache, ctypes.byref(pol))
    return rc, (pol.w_freq, pol.w_recency, pol.w_size, pol.freq_window)


def lora_cache_acquire(cache, adapter_id: int, rank: int, alpha: float = 1.0, pin: bool = True, queued_ids=None):
    """-> (status, slot, hit)"""
    keep, qp, nq = _ids(queued_ids)
    s, h = c_int32(-1), c_int32(0)
    rc = _lib.lora_cache_acquire(cache, adapter_id, rank, alpha, 1 if pin else 0, qp, nq, ctypes.byref(s), ctypes.byref(h))
    return rc, s.value, h.value


def lora_cache_score(cache, slot: int):
    v = ctypes.c_double(0.0)
    rc = _lib.lora_cache_score(cache, slot, ctypes.byref(v))
    return rc, v.value


def lora_cache_choose_victim(cache, rank: int = 0, queued_ids=None):
    keep, qp, nq = _ids(queued_ids)
    s = c_int32(-1)
    rc = _lib.lora_cache_choose_victim(cache, rank, qp, nq, ctypes.byref(s))
    return rc, s.value


def lora_cache_resident_bytes(cache):
    n = c_size_t(0)
    rc = _lib.lora_cache_resident_bytes(cache, ctypes.byref(n))
    return rc, n.value


def lora_cache_trim(cache, max_bytes: int, queued_ids=None):
    """-> (status, entries evicted)"""
    keep, qp, nq = _ids(queued_ids)
    n = c_int32(0)
    rc = _lib.lora_cache_trim(cache, max_bytes, qp, nq, ctypes.byref(n))
    return rc, n.value


# ---- scheduler (include/lora_sched.h) -----------------------------------------------------------

def lora_sched_wrs(input_len, output_len, rank, max_input, max_output, max_rank, a_input=0.0, b_output=0.0) -> float:
    return float(_lib.lora_sched_wrs(input_len, output_len, rank, max_input, max_output, max_rank, a_input, b_output))


def lora_sched_create(quota, boundaries, max_input, max_output, max_rank, tokens_per_rank, a_input=0.0, b_output=0.0):
    """-> (status, handle)"""
    q = np.ascontiguousarray(np.asarray(quota, dtype=np.int64))
    b = np.ascontiguousarray(np.asarray(boundaries, dtype=np.float64))
    cfg = lora_sched_config_t(int(q.size), q.ctypes.data_as(POINTER(c_int64)),
                              b.ctypes.data_as(POINTER(ctypes.c_double)) if b.size else None,
                              max_input, max_output, max_rank, tokens_per_rank, a_input, b_output)
    h = c_void_p()
    rc = _lib.lora_sched_create(ctypes.byref(cfg), ctypes.byref(h))
    return rc, h


def lora_sched_destroy(sched) -> int:
    return _lib.lora_sched_destroy(sched)


def lora_sched_submit(sched, req_id, input_len, output_len, adapter_id, rank):
    """-> (status, queue)"""
    q = c_int32(-1)
    rc = _lib.lora_sched_submit(sched, req_id, input_len, output_len, adapter_id, rank, ctypes.byref(q))
    return rc, q.value


def lora_sched_generate_batch(sched, cap: int = 4096):
    """-> (status, [request ids in admission order])"""
    ids = (c_int64 * max(1, cap))()
    n = c_int32(0)
    rc = _lib.lora_sched_generate_batch(sched, ids, cap, ctypes.byref(n))
    return rc, [int(ids[i]) for i in range(n.value)]


def lora_sched_finish(sched, req_id) -> int:
    return _lib.lora_sched_finish(sched, req_id)


def lora_sched_queue_state(sched, queue: int):
    """-> (status, free tokens, waiting requests)"""
    f, w = c_int64(0), c_int32(0)
    rc = _lib.lora_sched_queue_state(sched, queue, ctypes.byref(f), ctypes.byref(w))
    return rc, f.value, w.value


def lora_sched_waiting_adapters(sched, cap: int = 4096):
    ids = (c_int64 * max(1, cap))()
    n = c_int32(0)
    rc = _lib.lora_sched_waiting_adapters(sched, ids, cap, ctypes.byref(n))
    return rc, [int(ids[i]) for i in range(min(n.value, cap))]


def lora_sched_fit_queues(sizes, k_max: int = 4):
    """-> (status, K, [boundaries])"""
    x = np.ascontiguousarray(np.asarray(sizes, dtype=np.float64))
    k = c_int32(0)
    b = (ctypes.c_double * max(1, k_max))()
    rc = _lib.lora_sched_fit_queues(x.ctypes.data_as(POINTER(ctypes.c_double)), int(x.size), k_max, ctypes.byref(k), b)
    return rc, k.value, [float(b[i]) for i in range(max(0, k.value - 1))]


def lora_sched_min_quota(max_request_tokens, duration, slo, arrival_rate) -> int:
    return int(_lib.lora_sched_min_quota(max_request_tokens, duration, slo, arrival_rate))


def lora_sched_assign_quotas(total_tokens, least, weights):
    """-> (status, [quota per queue])"""
    l = np.ascontiguousarray(np.asarray(least, dtype=np.int64))
    w = np.ascontiguousarray(np.asarray(weights, dtype=np.float64))
    out = (c_int64 * max(1, int(l.size)))()
    rc = _lib.lora_sched_assign_quotas(total_tokens, l.ctypes.data_as(POINTER(c_int64)), w.ctypes.data_as(POINTER(ctypes.c_double)),
                                       int(l.size), out)
    return rc, [int(out[i]) for i in range(int(l.size))]


def lora_cache_slab(cache, layer: int, proj: int, slot: int):
    """-> (status, device address, bytes)"""
    p, n = c_void_p(), c_size_t()
    rc = _lib.lora_cache_slab(cache, layer, proj, slot, ctypes.byref(p), ctypes.byref(n))
    return rc, (p.value or 0), n.value


def _items(ptr, n):
    return [tuple(getattr(ptr[i], f) for f in ("tok_off", "n_tok", "slot", "rank", "a", "b")) for i in range(n)]


def lora_index(T: int, seg_offsets, seg_slot, seg_rank, mfma_min_tokens: int, counts_only: bool = False):
    """-> (status, dict of python lists with the same keys as the C struct); with counts_only the
    lists are not copied out, only their lengths (what a timing of the call itself wants)"""
    so, ss, sr = _i32(seg_offsets), _i32(seg_slot), _i32(seg_rank)
    w = lora_worklists_t()
    rc = _lib.lora_index(T, _ptr(so), _ptr(ss), _ptr(sr), len(ss), mfma_min_tokens, ctypes.byref(w))
    if rc != LORA_OK:
        return rc, None
    if counts_only:
        out = {"n_tok_list": w.n_tok_list, "n_tiles": w.n_tiles, "n_groups": w.n_groups}
        _lib.lora_worklists_free(ctypes.byref(w))
        return rc, out
    out = {
        "tok_list": [w.tok_list[i] for i in range(w.n_tok_list)],
        "tiles": _items(w.tiles, w.n_tiles),
        "groups": _items(w.groups, w.n_groups),
    }
    _lib.lora_worklists_free(ctypes.byref(w))
    return rc, out


def lora_plan_create(cache, T: int, seg_offsets, seg_slot, seg_rank, stream: int = 0):
    """-> (status, plan handle)"""
    so, ss, sr = _i32(seg_offsets), _i32(seg_slot), _i32(seg_rank)
    p = c_void_p()
    rc = _lib.lora_plan_create(cache, T, _ptr(so), _ptr(ss), _ptr(sr), len(ss), c_void_p(stream or None), ctypes.byref(p))
    return rc, p


def lora_plan_destroy(cache, plan) -> int:
    return _lib.lora_plan_destroy(cache, plan)


def lora_plan_info(plan):
    """-> (status, lora_plan_info_t)"""
    info = lora_plan_info_t()
    rc = _lib.lora_plan_info(plan, ctypes.byref(info))
    return rc, info


def lora_plan_dump(cache, plan, proj: int):
    """-> (status, units as a numpy record array with the fields of lora_plan_unit_t, tokens as an int32 array)"""
    nu, nt = c_int32(0), c_int32(0)
    rc = _lib.lora_plan_dump(cache, plan, proj, None, 0, ctypes.byref(nu), None, 0, ctypes.byref(nt))
    if rc != LORA_OK:
        return rc, None, None
    units = (lora_plan_unit_t * max(1, nu.value))()
    toks = np.zeros(max(1, nt.value), np.int32)
    rc = _lib.lora_plan_dump(cache, plan, proj, units, nu.value, ctypes.byref(nu), _ptr(toks), nt.value, ctypes.byref(nt))
    if rc != LORA_OK:
        return rc, None, None
    rec = np.frombuffer(units, dtype=np.dtype([(n, np.int32) for n in ("kind", "tok_off", "n_tok", "slot", "rank", "lo", "hi", "where")] + [("alpha", np.float32)]), count=nu.value).copy()
    return rc, rec, toks[: nt.value].copy()


def lora_apply_plan(cache, plan, layer: int, proj: int, x: int, base_out: int, scale: float, stream: int = 0) -> int:
    return _lib.lora_apply_plan(cache, plan, layer, proj, c_void_p(x or None), c_void_p(base_out or None), scale,
                                c_void_p(stream or None))


def lora_linear_workspace_bytes(cache, plan, proj: int):
    """-> (status, bytes)"""
    n = c_size_t(0)
    rc = _lib.lora_linear_workspace_bytes(cache, plan, proj, ctypes.byref(n))
    return rc, n.value


def lora_linear_plan(cache, plan, layer: int, proj: int, x: int, Wt: int, y: int, scale: float, stream: int = 0,
                     workspace: int = 0, workspace_bytes: int = 0) -> int:
    return _lib.lora_linear_plan(cache, plan, layer, proj, c_void_p(x or None), c_void_p(Wt or None), c_void_p(y or None), scale,
                                 c_void_p(workspace or None), workspace_bytes, c_void_p(stream or None))


def lora_apply_plan_static(cache, plan, layer: int, proj: int, x: int, base_out: int, scale: float, stream: int = 0) -> int:
    return _lib.lora_apply_plan_static(cache, plan, layer, proj, c_void_p(x or None), c_void_p(base_out or None), scale,
                                       c_void_p(stream or None))


LORA_STATIC_MAX_TOKENS = 4096


def make_descs(entries):
    """[(layer, proj, x device address, base_out device address), ...] -> C array for lora_apply_plan_multi."""
    arr = (lora_apply_desc_t * len(entries))()
    for i, (layer, proj, x, y) in enumerate(entries):
        arr[i] = lora_apply_desc_t(int(layer), int(proj), c_void_p(x or None), c_void_p(y or None))
    return arr


def lora_apply_plan_multi(cache, plan, descs, scale: float, stream: int = 0) -> int:
    return _lib.lora_apply_plan_multi(cache, plan, descs, len(descs), scale, c_void_p(stream or None))


def lora_apply(cache, layer: int, proj: int, x: int, base_out: int, T: int, seg_offsets, seg_slot, seg_rank,
               scale: float, stream: int = 0) -> int:
    so, ss, sr = _i32(seg_offsets), _i32(seg_slot), _i32(seg_rank)
    return _lib.lora_apply(cache, layer, proj, c_void_p(x or None), c_void_p(base_out or None), T, _ptr(so), _ptr(ss),
                           _ptr(sr), len(ss), scale, c_void_p(stream or None))


KERNEL_KINDS = ("mfma_reduce", "mfma_shrink", "gemv_shrink", "mfma_expand", "gemv_expand", "gemv_fused", "linear")


def lora_cache_set_timing(cache, on: int) -> int:
    return _lib.lora_cache_set_timing(cache, on)


def lora_cache_read_timing(cache):
    """-> (status, {kind: (milliseconds, launches)})"""
    ms = (ctypes.c_double * len(KERNEL_KINDS))()
    n = (c_int64 * len(KERNEL_KINDS))()
    rc = _lib.lora_cache_read_timing(cache, ms, n)
    return rc, {k: (ms[i], n[i]) for i, k in enumerate(KERNEL_KINDS)}


def lora_cache_check_fault(cache, stream: int = 0):
    """-> (status, fault)"""
    f = c_int32(0)
    rc = _lib.lora_cache_check_fault(cache, c_void_p(stream or None), ctypes.byref(f))
    return rc, f.value


def lora_cache_set_fencing(cache, on: int) -> int:
    return _lib.lora_cache_set_fencing(cache, on)
