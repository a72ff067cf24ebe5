"""ctypes binding of libelora.so -- argument marshalling only.

Function names and argument order follow include/elora.h.  Tensors are passed
as torch tensors on the GPU (PyTorch is used for device memory and streams
only); every step of the layer runs inside the library's HIP kernels.  There
is no fallback: importing this module without a built libelora.so raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("ELORA_LIB", os.path.join(_HERE, "libelora.so"))  # override: an alternative build

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `python -m paper_2507_01438_amd.build` "
        "(there is no non-HIP fallback for the batched LoRA linear layer)")

lib = ctypes.CDLL(LIB_PATH)

# ---- enums (include/elora.h) -------------------------------------------------
ELORA_OK = 0
(ELORA_E_NULL, ELORA_E_ALIGN, ELORA_E_DTYPE, ELORA_E_SHAPE, ELORA_E_RANK, ELORA_E_SLOT,
 ELORA_E_NOT_LOADED, ELORA_E_STORAGE, ELORA_E_SEGMENTS, ELORA_E_HIP) = range(1, 11)
ELORA_F32, ELORA_BF16 = 0, 1
ELORA_W_SAME, ELORA_W_INT4_G32, ELORA_W_INT8_G32 = 0, 1, 2
ELORA_PATH_GENERIC, ELORA_PATH_DECODE, ELORA_PATH_GEMM = 0, 1, 2

EXPORTED = [
    "elora_status_string", "elora_version", "elora_pool_storage_bytes", "elora_pool_create",
    "elora_pool_destroy", "elora_pool_storage_bytes_q8", "elora_pool_create_q8", "elora_pool_load_adapter", "elora_pool_load_adapters", "elora_pool_load_adapters_q8", "elora_pool_evict", "elora_pool_slot_info",
    "elora_pool_poll_error", "elora_workspace_bytes", "elora_workspace_bytes_w", "elora_linear_plan", "elora_batched_lora_linear",
    "elora_batched_lora_linear_group", "elora_linear_group_launches", "elora_batched_lora_linear_noalloc", "elora_force_path", "elora_profile_arm", "elora_profile_read", "elora_workspace_init",
    "elora_debug_spin_limit", "elora_debug_xcd_local", "elora_debug_k_rotate", "elora_debug_decode_wide", "elora_debug_decode_passes", "elora_debug_wait_limit_us", "elora_debug_w4_copy_rows",
    "elora_cache_create", "elora_cache_destroy", "elora_cache_acquire", "elora_cache_release", "elora_cache_lookup",
    "elora_cache_acquire_batch", "elora_cache_release_batch", "elora_cache_select",
    "elora_cache_drop", "elora_cache_stats", "elora_cache_reset_stats", "elora_cache_load_begin",
    "elora_cache_load_end", "elora_cache_batch_begin", "elora_cache_batch_end",
]


class elora_linear_desc_t(ctypes.Structure):
    _fields_ = [
        ("n_tokens", ctypes.c_int), ("d_in", ctypes.c_int), ("d_out", ctypes.c_int),
        ("dtype", ctypes.c_int), ("wfmt", ctypes.c_int),
        ("x", ctypes.c_void_p), ("W", ctypes.c_void_p), ("w_scales", ctypes.c_void_p), ("y", ctypes.c_void_p),
        ("pool", ctypes.c_void_p),
        ("adapter_idx", ctypes.c_void_p), ("seg_offsets", ctypes.c_void_p), ("seg_adapter", ctypes.c_void_p),
        ("n_segments", ctypes.c_int),
        ("scales", ctypes.c_void_p),
        ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
    ]


class elora_plan_t(ctypes.Structure):
    _fields_ = [("path", ctypes.c_int), ("n_launches", ctypes.c_int), ("split_k", ctypes.c_int),
                ("tile_rows", ctypes.c_int), ("tile_cols", ctypes.c_int), ("grid", ctypes.c_int)]


lib.elora_status_string.restype = ctypes.c_char_p
lib.elora_status_string.argtypes = [ctypes.c_int]
lib.elora_version.restype = ctypes.c_int
lib.elora_pool_storage_bytes.restype = ctypes.c_size_t
lib.elora_pool_storage_bytes.argtypes = [ctypes.c_int] * 5
lib.elora_pool_create.restype = ctypes.c_int
lib.elora_pool_create.argtypes = [ctypes.c_int] * 5 + [ctypes.c_void_p, ctypes.c_size_t, ctypes.POINTER(ctypes.c_void_p)]
lib.elora_pool_storage_bytes_q8.restype = ctypes.c_size_t
lib.elora_pool_storage_bytes_q8.argtypes = [ctypes.c_int] * 4
lib.elora_pool_create_q8.restype = ctypes.c_int
lib.elora_pool_create_q8.argtypes = [ctypes.c_int] * 4 + [ctypes.c_void_p, ctypes.c_size_t, ctypes.POINTER(ctypes.c_void_p)]
lib.elora_pool_destroy.restype = ctypes.c_int
lib.elora_pool_destroy.argtypes = [ctypes.c_void_p]
lib.elora_pool_load_adapter.restype = ctypes.c_int
lib.elora_pool_load_adapter.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_float,
                                        ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p]
lib.elora_pool_load_adapters.restype = ctypes.c_int
lib.elora_pool_load_adapters.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                         ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
lib.elora_pool_load_adapters_q8.restype = ctypes.c_int
lib.elora_pool_load_adapters_q8.argtypes = [ctypes.c_void_p, ctypes.c_int] + [ctypes.c_void_p] * 8
lib.elora_pool_evict.restype = ctypes.c_int
lib.elora_pool_evict.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p]
lib.elora_pool_slot_info.restype = ctypes.c_int
lib.elora_pool_slot_info.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_float)]
lib.elora_pool_poll_error.restype = ctypes.c_int
lib.elora_pool_poll_error.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.POINTER(ctypes.c_int),
                                      ctypes.POINTER(ctypes.c_int), ctypes.c_void_p]
lib.elora_workspace_bytes.restype = ctypes.c_size_t
lib.elora_workspace_bytes.argtypes = [ctypes.c_int] * 4
lib.elora_workspace_bytes_w.restype = ctypes.c_size_t
lib.elora_workspace_bytes_w.argtypes = [ctypes.c_int] * 5
lib.elora_linear_plan.restype = ctypes.c_int
lib.elora_linear_plan.argtypes = [ctypes.POINTER(elora_linear_desc_t), ctypes.POINTER(elora_plan_t)]
lib.elora_batched_lora_linear.restype = ctypes.c_int
lib.elora_batched_lora_linear.argtypes = [ctypes.POINTER(elora_linear_desc_t), ctypes.c_void_p]
lib.elora_batched_lora_linear_noalloc.restype = ctypes.c_int
lib.elora_batched_lora_linear_noalloc.argtypes = [ctypes.POINTER(elora_linear_desc_t), ctypes.c_void_p]
lib.elora_batched_lora_linear_group.restype = ctypes.c_int
lib.elora_batched_lora_linear_group.argtypes = [ctypes.POINTER(elora_linear_desc_t), ctypes.c_int, ctypes.c_void_p]
lib.elora_linear_group_launches.restype = ctypes.c_int
lib.elora_linear_group_launches.argtypes = [ctypes.POINTER(elora_linear_desc_t), ctypes.c_int, ctypes.POINTER(ctypes.c_int)]
lib.elora_force_path.restype = ctypes.c_int
lib.elora_force_path.argtypes = [ctypes.c_int]


lib.elora_workspace_init.restype = ctypes.c_int
lib.elora_workspace_init.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
lib.elora_debug_spin_limit.restype = ctypes.c_int
lib.elora_debug_spin_limit.argtypes = [ctypes.c_int]
lib.elora_debug_xcd_local.restype = ctypes.c_int
lib.elora_debug_xcd_local.argtypes = [ctypes.c_int]
lib.elora_debug_wait_limit_us.restype = ctypes.c_int
lib.elora_debug_wait_limit_us.argtypes = [ctypes.c_int]
lib.elora_debug_w4_copy_rows.restype = ctypes.c_int
lib.elora_debug_w4_copy_rows.argtypes = [ctypes.c_int]
lib.elora_debug_decode_passes.restype = ctypes.c_int
lib.elora_debug_decode_passes.argtypes = [ctypes.c_int]
lib.elora_debug_decode_wide.restype = ctypes.c_int
lib.elora_debug_decode_wide.argtypes = [ctypes.c_int]
lib.elora_debug_k_rotate.restype = ctypes.c_int
lib.elora_debug_k_rotate.argtypes = [ctypes.c_int]
lib.elora_profile_arm.restype = ctypes.c_int
lib.elora_profile_arm.argtypes = [ctypes.c_int]
lib.elora_profile_read.restype = ctypes.c_int
lib.elora_profile_read.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_int, ctypes.POINTER(ctypes.c_int)]
_ip = ctypes.POINTER(ctypes.c_int)
_llp = ctypes.POINTER(ctypes.c_longlong)
lib.elora_cache_create.restype = ctypes.c_int
lib.elora_cache_create.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_void_p)]
lib.elora_cache_destroy.restype = ctypes.c_int
lib.elora_cache_destroy.argtypes = [ctypes.c_void_p]
lib.elora_cache_acquire.restype = ctypes.c_int
lib.elora_cache_acquire.argtypes = [ctypes.c_void_p, ctypes.c_int, _ip, _ip, _ip]
lib.elora_cache_release.restype = ctypes.c_int
lib.elora_cache_release.argtypes = [ctypes.c_void_p, ctypes.c_int]
lib.elora_cache_acquire_batch.restype = ctypes.c_int
lib.elora_cache_acquire_batch.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p,
                                          ctypes.c_void_p, _ip]
lib.elora_cache_release_batch.restype = ctypes.c_int
lib.elora_cache_release_batch.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int]
lib.elora_cache_select.restype = ctypes.c_int
lib.elora_cache_select.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, _ip, _ip]
lib.elora_cache_lookup.restype = ctypes.c_int
lib.elora_cache_lookup.argtypes = [ctypes.c_void_p, ctypes.c_int, _ip]
lib.elora_cache_drop.restype = ctypes.c_int
lib.elora_cache_drop.argtypes = [ctypes.c_void_p, ctypes.c_int]
lib.elora_cache_stats.restype = ctypes.c_int
lib.elora_cache_stats.argtypes = [ctypes.c_void_p, _llp, _llp, _llp]
lib.elora_cache_reset_stats.restype = ctypes.c_int
lib.elora_cache_reset_stats.argtypes = [ctypes.c_void_p]
for _name in ("elora_cache_load_begin", "elora_cache_load_end", "elora_cache_batch_begin", "elora_cache_batch_end"):
    getattr(lib, _name).restype = ctypes.c_int
    getattr(lib, _name).argtypes = [ctypes.c_void_p, _ip, ctypes.c_int, ctypes.c_void_p]


class EloraError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = int(status)
        super().__init__(f"{where}: {elora_status_string(status)} (status {status})")


def _check(status: int, where: str) -> None:
    if status != ELORA_OK:
        raise EloraError(status, where)


def _ptr(t) -> Optional[int]:
    """Device/host address of a tensor, an int address, or None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


# ---- same-name wrappers ---------------------------------------------------------

def elora_status_string(status: int) -> str:
    return lib.elora_status_string(int(status)).decode()


def elora_version() -> int:
    return int(lib.elora_version())


def elora_pool_storage_bytes(d_in: int, d_out: int, max_rank: int, capacity: int, dtype: int) -> int:
    return int(lib.elora_pool_storage_bytes(d_in, d_out, max_rank, capacity, dtype))


def elora_pool_create(d_in, d_out, max_rank, capacity, dtype, dev_storage, storage_bytes) -> int:
    """Returns the opaque pool handle (an address)."""
    out = ctypes.c_void_p()
    _check(lib.elora_pool_create(d_in, d_out, max_rank, capacity, dtype, _ptr(dev_storage), storage_bytes,
                                 ctypes.byref(out)), "elora_pool_create")
    return out.value


def elora_pool_storage_bytes_q8(d_in: int, d_out: int, max_rank: int, capacity: int) -> int:
    return int(lib.elora_pool_storage_bytes_q8(d_in, d_out, max_rank, capacity))


def elora_pool_create_q8(d_in, d_out, max_rank, capacity, dev_storage, storage_bytes) -> int:
    out = ctypes.c_void_p()
    _check(lib.elora_pool_create_q8(d_in, d_out, max_rank, capacity, _ptr(dev_storage), storage_bytes, ctypes.byref(out)),
           "elora_pool_create_q8")
    return out.value


def elora_pool_destroy(pool: int) -> None:
    _check(lib.elora_pool_destroy(pool), "elora_pool_destroy")


def elora_pool_load_adapter(pool, slot, rank, scale, A, B, src_on_device, stream=None) -> None:
    _check(lib.elora_pool_load_adapter(pool, slot, rank, scale, _ptr(A), _ptr(B), int(src_on_device),
                                       _stream(stream)), "elora_pool_load_adapter")


def elora_pool_load_adapters(pool, slots, ranks, scales, A, B, stream=None) -> None:
    """Sequences of equal length; A and B hold tensors (device or pinned host) or addresses."""
    n = len(slots)
    sl = (ctypes.c_int * n)(*[int(v) for v in slots])
    rk = (ctypes.c_int * n)(*[int(v) for v in ranks])
    sc = (ctypes.c_float * n)(*[float(v) for v in scales])
    pa = (ctypes.c_void_p * n)(*[_ptr(t) for t in A])
    pb = (ctypes.c_void_p * n)(*[_ptr(t) for t in B])
    _check(lib.elora_pool_load_adapters(pool, n, sl, rk, sc, pa, pb, _stream(stream)), "elora_pool_load_adapters")


def elora_pool_load_adapters_q8(pool, slots, ranks, scales, A_codes, A_scales, B_codes, B_scales, stream=None) -> None:
    """Sequences of equal length; the last four hold tensors (device or pinned host) or addresses."""
    n = len(slots)
    sl = (ctypes.c_int * n)(*[int(v) for v in slots])
    rk = (ctypes.c_int * n)(*[int(v) for v in ranks])
    sc = (ctypes.c_float * n)(*[float(v) for v in scales])
    ptrs = [(ctypes.c_void_p * n)(*[_ptr(t) for t in seq]) for seq in (A_codes, A_scales, B_codes, B_scales)]
    _check(lib.elora_pool_load_adapters_q8(pool, n, sl, rk, sc, *ptrs, _stream(stream)), "elora_pool_load_adapters_q8")


def elora_pool_evict(pool, slot, stream=None) -> None:
    _check(lib.elora_pool_evict(pool, slot, _stream(stream)), "elora_pool_evict")


def elora_pool_slot_info(pool, slot):
    r, s = ctypes.c_int(), ctypes.c_float()
    _check(lib.elora_pool_slot_info(pool, slot, ctypes.byref(r), ctypes.byref(s)), "elora_pool_slot_info")
    return r.value, s.value


def elora_pool_poll_error(pool, clear: bool = True, stream=None):
    """(n_bad_rows, first_bad_row); synchronises the stream."""
    n, f = ctypes.c_int(), ctypes.c_int()
    _check(lib.elora_pool_poll_error(pool, int(clear), ctypes.byref(n), ctypes.byref(f), _stream(stream)),
           "elora_pool_poll_error")
    return n.value, f.value


def elora_workspace_bytes(n_tokens_max: int, d_in: int, d_out: int, max_rank: int) -> int:
    return int(lib.elora_workspace_bytes(n_tokens_max, d_in, d_out, max_rank))


def elora_workspace_bytes_w(n_tokens_max: int, d_in: int, d_out: int, max_rank: int, wfmt: int) -> int:
    return int(lib.elora_workspace_bytes_w(n_tokens_max, d_in, d_out, max_rank, wfmt))


def make_desc(*, n_tokens, d_in, d_out, dtype, x, W, y, workspace, workspace_bytes, wfmt=ELORA_W_SAME,
              w_scales=None, pool=None, adapter_idx=None, seg_offsets=None, seg_adapter=None, n_segments=0,
              scales=None) -> elora_linear_desc_t:
    d = elora_linear_desc_t()
    d.n_tokens, d.d_in, d.d_out, d.dtype, d.wfmt = n_tokens, d_in, d_out, dtype, wfmt
    d.x, d.W, d.w_scales, d.y = _ptr(x), _ptr(W), _ptr(w_scales), _ptr(y)
    d.pool = pool
    d.adapter_idx, d.seg_offsets, d.seg_adapter = _ptr(adapter_idx), _ptr(seg_offsets), _ptr(seg_adapter)
    d.n_segments = n_segments
    d.scales = _ptr(scales)
    d.workspace, d.workspace_bytes = _ptr(workspace), workspace_bytes
    return d


def elora_linear_plan(desc: elora_linear_desc_t) -> elora_plan_t:
    plan = elora_plan_t()
    _check(lib.elora_linear_plan(ctypes.byref(desc), ctypes.byref(plan)), "elora_linear_plan")
    return plan


def elora_batched_lora_linear(desc: elora_linear_desc_t, stream=None) -> None:
    _check(lib.elora_batched_lora_linear(ctypes.byref(desc), _stream(stream)), "elora_batched_lora_linear")


def elora_batched_lora_linear_noalloc(desc: elora_linear_desc_t, stream=None) -> None:
    _check(lib.elora_batched_lora_linear_noalloc(ctypes.byref(desc), _stream(stream)), "elora_batched_lora_linear_noalloc")


def desc_array(descs):
    """A contiguous C array of descriptors (for the group calls); keep it alive while the call is enqueued."""
    arr = (elora_linear_desc_t * len(descs))()
    for i, d in enumerate(descs):
        ctypes.memmove(ctypes.byref(arr[i]), ctypes.byref(d), ctypes.sizeof(elora_linear_desc_t))
    return arr


def elora_batched_lora_linear_group(descs, stream=None) -> None:
    arr = descs if isinstance(descs, ctypes.Array) else desc_array(descs)
    _check(lib.elora_batched_lora_linear_group(arr, len(arr), _stream(stream)), "elora_batched_lora_linear_group")


def elora_linear_group_launches(descs) -> int:
    arr = descs if isinstance(descs, ctypes.Array) else desc_array(descs)
    n = ctypes.c_int()
    _check(lib.elora_linear_group_launches(arr, len(arr), ctypes.byref(n)), "elora_linear_group_launches")
    return n.value


def elora_force_path(path: int) -> None:
    _check(lib.elora_force_path(path), "elora_force_path")


def elora_workspace_init(workspace, workspace_bytes: int, stream=None) -> None:
    _check(lib.elora_workspace_init(_ptr(workspace), workspace_bytes, _stream(stream)), "elora_workspace_init")


def elora_debug_spin_limit(limit: int) -> None:
    _check(lib.elora_debug_spin_limit(int(limit)), "elora_debug_spin_limit")


def elora_debug_xcd_local(mode: int) -> None:
    _check(lib.elora_debug_xcd_local(int(mode)), "elora_debug_xcd_local")


def elora_debug_w4_copy_rows(rows: int) -> None:
    _check(lib.elora_debug_w4_copy_rows(int(rows)), "elora_debug_w4_copy_rows")


def elora_debug_wait_limit_us(us: int) -> None:
    _check(lib.elora_debug_wait_limit_us(int(us)), "elora_debug_wait_limit_us")


def elora_debug_decode_passes(mode: int) -> None:
    _check(lib.elora_debug_decode_passes(int(mode)), "elora_debug_decode_passes")


def elora_debug_decode_wide(mode: int) -> None:
    _check(lib.elora_debug_decode_wide(int(mode)), "elora_debug_decode_wide")


def elora_debug_k_rotate(on: int) -> None:
    _check(lib.elora_debug_k_rotate(int(on)), "elora_debug_k_rotate")


def elora_profile_arm(n_calls: int) -> None:
    _check(lib.elora_profile_arm(int(n_calls)), "elora_profile_arm")


def elora_profile_read(n: int):
    """Elapsed milliseconds of the dominant kernel of each armed call that has run (list of floats)."""
    buf = (ctypes.c_float * max(n, 1))()
    got = ctypes.c_int()
    _check(lib.elora_profile_read(buf, int(n), ctypes.byref(got)), "elora_profile_read")
    return [float(buf[i]) for i in range(got.value)]


# ---- small holders that keep device memory alive (no arithmetic) ----------------------

_TORCH_DTYPE = {ELORA_F32: torch.float32, ELORA_BF16: torch.bfloat16}


# ---- adapter cache (Sec. 3.3 / 4.2): argument marshalling only ----------------------

ELORA_E_NOT_LOADED = 7
ELORA_E_BUSY = 11


def elora_cache_create(capacity: int) -> int:
    out = ctypes.c_void_p()
    _check(lib.elora_cache_create(int(capacity), ctypes.byref(out)), "elora_cache_create")
    return out.value


def elora_cache_destroy(cache: int) -> None:
    _check(lib.elora_cache_destroy(cache), "elora_cache_destroy")


def elora_cache_acquire(cache: int, adapter_id: int):
    """(slot, hit, evicted adapter id or -1)"""
    slot, hit, ev = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
    _check(lib.elora_cache_acquire(cache, int(adapter_id), ctypes.byref(slot), ctypes.byref(hit), ctypes.byref(ev)),
           "elora_cache_acquire")
    return slot.value, bool(hit.value), ev.value


def elora_cache_release(cache: int, adapter_id: int) -> None:
    _check(lib.elora_cache_release(cache, int(adapter_id)), "elora_cache_release")


def elora_cache_acquire_batch(cache: int, adapter_ids: np.ndarray, slots: np.ndarray, miss_ids: np.ndarray,
                              miss_slots: np.ndarray) -> int:
    """Host int32 arrays of the same length (adapter_ids in; the others out).  Returns the number of misses."""
    n = int(adapter_ids.shape[0])
    for a in (adapter_ids, slots, miss_ids, miss_slots):
        assert a.dtype == np.int32 and a.flags.c_contiguous and a.shape[0] >= n
    n_miss = ctypes.c_int()
    _check(lib.elora_cache_acquire_batch(cache, adapter_ids.ctypes.data, n, slots.ctypes.data, miss_ids.ctypes.data,
                                         miss_slots.ctypes.data, ctypes.byref(n_miss)), "elora_cache_acquire_batch")
    return n_miss.value


def elora_cache_release_batch(cache: int, adapter_ids: np.ndarray) -> None:
    assert adapter_ids.dtype == np.int32 and adapter_ids.flags.c_contiguous
    _check(lib.elora_cache_release_batch(cache, adapter_ids.ctypes.data, int(adapter_ids.shape[0])),
           "elora_cache_release_batch")


def elora_cache_select(cache: int, explicit_id: int, scores: Optional[np.ndarray], k: int):
    """(chosen adapter id, resident?)  scores: host float32 array or None when explicit_id >= 0."""
    chosen, resident = ctypes.c_int(), ctypes.c_int()
    if scores is not None:
        assert scores.dtype == np.float32 and scores.flags.c_contiguous
    _check(lib.elora_cache_select(cache, int(explicit_id), None if scores is None else scores.ctypes.data,
                                  0 if scores is None else int(scores.shape[0]), int(k), ctypes.byref(chosen),
                                  ctypes.byref(resident)), "elora_cache_select")
    return chosen.value, bool(resident.value)


def elora_cache_lookup(cache: int, adapter_id: int) -> int:
    slot = ctypes.c_int()
    _check(lib.elora_cache_lookup(cache, int(adapter_id), ctypes.byref(slot)), "elora_cache_lookup")
    return slot.value


def elora_cache_drop(cache: int, adapter_id: int) -> None:
    _check(lib.elora_cache_drop(cache, int(adapter_id)), "elora_cache_drop")


def elora_cache_stats(cache: int):
    """(hits, requests, evictions)"""
    h, r, e = ctypes.c_longlong(), ctypes.c_longlong(), ctypes.c_longlong()
    _check(lib.elora_cache_stats(cache, ctypes.byref(h), ctypes.byref(r), ctypes.byref(e)), "elora_cache_stats")
    return h.value, r.value, e.value


def elora_cache_reset_stats(cache: int) -> None:
    _check(lib.elora_cache_reset_stats(cache), "elora_cache_reset_stats")


def _int_array(values):
    values = [int(v) for v in values]
    return (ctypes.c_int * len(values))(*values), len(values)


def elora_cache_load_begin(cache: int, slots, copy_stream) -> None:
    arr, n = _int_array(slots)
    _check(lib.elora_cache_load_begin(cache, arr, n, _stream(copy_stream)), "elora_cache_load_begin")


def elora_cache_load_end(cache: int, slots, copy_stream) -> None:
    arr, n = _int_array(slots)
    _check(lib.elora_cache_load_end(cache, arr, n, _stream(copy_stream)), "elora_cache_load_end")


def elora_cache_batch_begin(cache: int, slots, compute_stream=None) -> None:
    arr, n = _int_array(slots)
    _check(lib.elora_cache_batch_begin(cache, arr, n, _stream(compute_stream)), "elora_cache_batch_begin")


def elora_cache_batch_end(cache: int, slots, compute_stream=None) -> None:
    arr, n = _int_array(slots)
    _check(lib.elora_cache_batch_end(cache, arr, n, _stream(compute_stream)), "elora_cache_batch_end")


class AdapterPool:
    """Device storage (a torch byte tensor) plus the library's pool handle."""

    def __init__(self, d_in, d_out, max_rank, capacity, dtype, device="cuda:0", q8=False):
        """q8: the adapters stay in 8-bit blocks (elora_pool_create_q8; dtype must be bf16)."""
        self.d_in, self.d_out, self.max_rank, self.capacity, self.dtype, self.q8 = d_in, d_out, max_rank, capacity, dtype, q8
        self.nbytes = (elora_pool_storage_bytes_q8(d_in, d_out, max_rank, capacity) if q8 else
                       elora_pool_storage_bytes(d_in, d_out, max_rank, capacity, dtype))
        if self.nbytes == 0:
            raise EloraError(ELORA_E_SHAPE, "elora_pool_storage_bytes")
        self.storage = torch.empty(self.nbytes, dtype=torch.uint8, device=device)
        if q8:
            assert dtype == ELORA_BF16
            self.handle = elora_pool_create_q8(d_in, d_out, max_rank, capacity, self.storage, self.nbytes)
        else:
            self.handle = elora_pool_create(d_in, d_out, max_rank, capacity, dtype, self.storage, self.nbytes)

    def load(self, slot, A, B, scale, stream=None):
        """A [rank, d_in], B [d_out, rank]: torch tensors (device or host, contiguous) of the pool's dtype."""
        assert A.is_contiguous() and B.is_contiguous()
        assert A.is_cuda == B.is_cuda
        elora_pool_load_adapter(self.handle, slot, A.shape[0], float(scale), A, B, A.is_cuda, stream)

    def evict(self, slot, stream=None):
        elora_pool_evict(self.handle, slot, stream)

    def poll_error(self, clear=True, stream=None):
        return elora_pool_poll_error(self.handle, clear, stream)

    def close(self):
        if self.handle is not None:
            elora_pool_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class LoraLinear:
    """Pre-allocated workspace + descriptor assembly for repeated calls on one layer."""

    def __init__(self, d_in, d_out, dtype, pool: Optional[AdapterPool], n_tokens_max, device="cuda:0", wfmt=ELORA_W_SAME):
        self.d_in, self.d_out, self.dtype, self.pool = d_in, d_out, dtype, pool
        self.n_tokens_max = n_tokens_max
        self.ws_bytes = elora_workspace_bytes_w(n_tokens_max, d_in, d_out, pool.max_rank if pool else 1, wfmt)
        self.workspace = torch.empty(self.ws_bytes, dtype=torch.uint8, device=device)
        elora_workspace_init(self.workspace, self.ws_bytes)

    def desc(self, x, W, y, *, adapter_idx=None, seg_offsets=None, seg_adapter=None, scales=None,
             wfmt=ELORA_W_SAME, w_scales=None) -> elora_linear_desc_t:
        n_tokens = x.shape[0]
        assert n_tokens <= self.n_tokens_max
        return make_desc(
            n_tokens=n_tokens, d_in=self.d_in, d_out=self.d_out, dtype=self.dtype, wfmt=wfmt, x=x, W=W,
            w_scales=w_scales, y=y, pool=self.pool.handle if self.pool else None, adapter_idx=adapter_idx,
            seg_offsets=seg_offsets, seg_adapter=seg_adapter,
            n_segments=0 if seg_adapter is None else int(seg_adapter.shape[0]), scales=scales,
            workspace=self.workspace, workspace_bytes=self.ws_bytes)

    def __call__(self, x, W, y, stream=None, **kw):
        d = self.desc(x, W, y, **kw)
        elora_batched_lora_linear(d, stream)
        return y
