"""ctypes binding of libslora_hip.so: argument marshalling only, same names as include/slora.h.

Every step of the path (page scatter/gather, scheduling, shrink, expand) runs inside the
library.  There is no fallback: if the library is missing, loading raises.
Device pointers are passed as integers (e.g. torch.Tensor.data_ptr()); streams as integers
(torch.cuda.Stream.cuda_stream) or 0/None for the default stream.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

F16, BF16 = 0, 1
OK, EINVAL, ERANGE, EBUSY, ENOENT, ESEG, EHIP, ENOMEM = 0, -1, -2, -3, -4, -5, -6, -7
MAX_MULTI = 8
STATIC_SCRATCH_BYTES = 64 << 20
PLAN_INFO_N = 13
POOL_STATS_N = 3
PLAN_INFO_KEYS = ("tokens", "groups", "groups_vec", "groups_mfma", "vec_shrink_items", "vec_expand_items",
                  "mfma_shrink_items", "mfma_expand_items", "v_stride", "sum_rank", "split_tiles",
                  "scratch_bytes_per_slot", "groups_fused")

LIB_PATH = os.environ.get("SLORA_LIB") or os.path.join(os.path.dirname(os.path.abspath(__file__)), "libslora_hip.so")
_lib = None


class SloraError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"slora error {code}: {msg}")
        self.code = code


def lib() -> C.CDLL:
    """Load the HIP library (built in-tree by paper_2311_03285_amd/build.py)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: run `python -m paper_2311_03285_amd.build` "
                                    "(there is no CPU fallback)")
        try:
            # PyTorch ships its own HIP runtime; load it first so that this library binds to the
            # same one (two runtimes in a process do not see each other's device state)
            import torch  # noqa: F401
        except ImportError:
            pass
        L = C.CDLL(LIB_PATH)
        vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
        sig = {
            "slora_last_error": (C.c_char_p, []),
            "slora_pool_init": (i32, [C.POINTER(vp), i32, i64, i32, vp, i32, i32]),
            "slora_pool_destroy": (i32, [vp]),
            "slora_pool_stats": (i32, [vp, vp, i32]),
            "slora_pool_mark_kv": (i32, [vp, vp, i64, i32]),
            "slora_pool_write_pages": (i32, [vp, vp, i64, vp, i32, vp]),
            "slora_adapter_load": (i32, [vp, i32, i32, vp, i64]),
            "slora_adapter_unload": (i32, [vp, i32]),
            "slora_adapter_gather": (i32, [vp, i32, i32, i32, vp, vp]),
            "slora_pool_free_pages": (i32, [vp, vp]),
            "slora_pool_alloc_kv": (i32, [vp, i64, vp]),
            "slora_adapter_alloc": (i32, [vp, i32, i32, vp]),
            "slora_adapter_upload": (i32, [vp, i32, vp, vp]),
            "slora_batch_plan": (i32, [vp, C.POINTER(vp), vp, i32, vp, i32]),
            "slora_plan_destroy": (i32, [vp]),
            "slora_plan_info": (i32, [vp, vp, i32]),
            "slora_lora_apply": (i32, [vp, i32, vp, vp, vp]),
            "slora_lora_apply_multi": (i32, [vp, i32, vp, vp, vp, vp]),
            "slora_lora_apply_multi_y16": (i32, [vp, i32, vp, vp, vp, vp]),
            "slora_lora_apply_multi_static": (i32, [vp, i32, vp, vp, vp, vp]),
            "slora_lora_expand_y16": (i32, [vp, i32, vp, vp, vp]),
            "slora_lora_shrink": (i32, [vp, i32, vp, vp, vp]),
            "slora_lora_expand": (i32, [vp, i32, vp, vp, vp]),
            "slora_lora_shrink_expand": (i32, [vp, i32, vp, vp, vp, i32, i32, vp, vp]),
            "slora_set_option": (i32, [vp, C.c_char_p, i64]),
        }
        for name, (res, args) in sig.items():
            f = getattr(L, name)
            f.restype, f.argtypes = res, args
        _lib = L
    return _lib


def last_error() -> str:
    return lib().slora_last_error().decode()


def _check(rc: int) -> None:
    if rc != OK:
        raise SloraError(rc, last_error())


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else C.c_void_p(a.ctypes.data)


def _stream(s) -> Optional[int]:
    if s is None:
        return None
    return int(getattr(s, "cuda_stream", s)) or None


def _ptr_array(ptrs: Sequence[int]):
    return (C.c_void_p * len(ptrs))(*[C.c_void_p(int(p)) for p in ptrs])


# ---- the C calls, one to one ---------------------------------------------------------------
def pool_init(page_H: int, n_pages: int, dtype: int, dev_base: Optional[int], n_slots: int = 1,
              max_rank: int = 128) -> C.c_void_p:
    h = C.c_void_p()
    _check(lib().slora_pool_init(C.byref(h), page_H, n_pages, dtype, dev_base or None, n_slots, max_rank))
    return h


def pool_destroy(pool) -> None:
    _check(lib().slora_pool_destroy(pool))


def pool_stats(pool) -> dict:
    out = np.zeros(POOL_STATS_N, dtype=np.int64)
    _check(lib().slora_pool_stats(pool, _ptr(out), POOL_STATS_N))
    return dict(zip(("sets_made", "allocations", "idle_sets"), (int(v) for v in out)))


def pool_mark_kv(pool, page_idx, owned: bool = True) -> None:
    a = _i32(page_idx)
    _check(lib().slora_pool_mark_kv(pool, _ptr(a), a.size, 1 if owned else 0))


def pool_write_pages(pool, page_idx, src, src_on_device: bool, stream=None) -> None:
    """src: device pointer (int) if src_on_device, else a host numpy array of 16-bit patterns."""
    a = _i32(page_idx)
    if src_on_device:
        p = C.c_void_p(int(src))
    else:
        src = np.ascontiguousarray(src, dtype=np.uint16)
        p = _ptr(src)
    _check(lib().slora_pool_write_pages(pool, _ptr(a), a.size, p, 1 if src_on_device else 0, _stream(stream)))


def adapter_load(pool, adapter_id: int, rank: int, page_idx) -> None:
    a = _i32(page_idx).reshape(-1)
    _check(lib().slora_adapter_load(pool, adapter_id, rank, _ptr(a) if a.size else None, a.size))


def pool_free_pages(pool) -> int:
    n = np.zeros(1, dtype=np.int64)
    _check(lib().slora_pool_free_pages(pool, _ptr(n)))
    return int(n[0])


def pool_alloc_kv(pool, n: int) -> np.ndarray:
    """n free pages become KV pages; returns their indices."""
    out = np.zeros(max(int(n), 1), dtype=np.int32)
    _check(lib().slora_pool_alloc_kv(pool, int(n), _ptr(out)))
    return out[:int(n)]


def adapter_alloc(pool, adapter_id: int, rank: int, n_slots: int) -> np.ndarray:
    """Make the adapter resident on pages the library chooses; returns them as [n_slots, 2, rank]."""
    out = np.zeros(max(n_slots * 2 * rank, 1), dtype=np.int32)
    _check(lib().slora_adapter_alloc(pool, adapter_id, rank, _ptr(out)))
    return out[:n_slots * 2 * rank].reshape(n_slots, 2, rank)


def adapter_upload(pool, adapter_id: int, weights: int, stream=None) -> None:
    """weights: address of pinned host or device memory laid out [slot][A columns][B rows][H]."""
    _check(lib().slora_adapter_upload(pool, adapter_id, C.c_void_p(int(weights)) if weights else None,
                                      _stream(stream)))


def adapter_unload(pool, adapter_id: int) -> None:
    _check(lib().slora_adapter_unload(pool, adapter_id))


def adapter_gather(pool, adapter_id: int, slot: int, which: int, dev_out: int, stream=None) -> None:
    _check(lib().slora_adapter_gather(pool, adapter_id, slot, which, dev_out or None, _stream(stream)))


def batch_plan(pool, token_adapter_ids, seg_offsets=None) -> C.c_void_p:
    ids = _i32(token_adapter_ids)
    seg = None if seg_offsets is None else _i32(seg_offsets)
    h = C.c_void_p()
    _check(lib().slora_batch_plan(pool, C.byref(h), _ptr(ids) if ids.size else None, ids.size, _ptr(seg),
                                  0 if seg is None else seg.size - 1))
    return h


def plan_destroy(plan) -> None:
    _check(lib().slora_plan_destroy(plan))


def plan_info(plan) -> dict:
    out = np.zeros(PLAN_INFO_N, dtype=np.int64)
    _check(lib().slora_plan_info(plan, _ptr(out), PLAN_INFO_N))
    return dict(zip(PLAN_INFO_KEYS, (int(v) for v in out)))


def lora_apply(plan, slot: int, x: int, y: int, stream=None) -> None:
    _check(lib().slora_lora_apply(plan, slot, x or None, y or None, _stream(stream)))


def lora_apply_multi(plan, slots, xs: Sequence[int], ys: Sequence[int], stream=None) -> None:
    s = _i32(slots)
    _check(lib().slora_lora_apply_multi(plan, s.size, _ptr(s), _ptr_array(xs), _ptr_array(ys), _stream(stream)))


def lora_apply_multi_static(plan, slots, xs: Sequence[int], ys: Sequence[int], stream=None) -> None:
    """As lora_apply_multi, with v in the library's static scratch: allocates nothing."""
    s = _i32(slots)
    _check(lib().slora_lora_apply_multi_static(plan, s.size, _ptr(s), _ptr_array(xs), _ptr_array(ys), _stream(stream)))


def lora_apply_multi_y16(plan, slots, xs: Sequence[int], ys: Sequence[int], stream=None) -> None:
    """As lora_apply_multi, with every y of the pool's 16-bit storage type."""
    s = _i32(slots)
    _check(lib().slora_lora_apply_multi_y16(plan, s.size, _ptr(s), _ptr_array(xs), _ptr_array(ys), _stream(stream)))


def lora_expand_y16(plan, slots, ys: Sequence[int], stream=None) -> None:
    s = _i32(slots)
    _check(lib().slora_lora_expand_y16(plan, s.size, _ptr(s), _ptr_array(ys), _stream(stream)))


def lora_shrink(plan, slots, xs: Sequence[int], stream=None) -> None:
    s = _i32(slots)
    _check(lib().slora_lora_shrink(plan, s.size, _ptr(s), _ptr_array(xs), _stream(stream)))


def lora_expand(plan, slots, ys: Sequence[int], stream=None) -> None:
    s = _i32(slots)
    _check(lib().slora_lora_expand(plan, s.size, _ptr(s), _ptr_array(ys), _stream(stream)))


def lora_shrink_expand(pool, slot: int, x: int, token_adapter_ids, seg_offsets, y: int, stream=None) -> None:
    ids = _i32(token_adapter_ids)
    seg = None if seg_offsets is None else _i32(seg_offsets)
    _check(lib().slora_lora_shrink_expand(pool, slot, x or None, _ptr(ids) if ids.size else None, _ptr(seg),
                                          0 if seg is None else seg.size - 1, ids.size, y or None,
                                          _stream(stream)))


def set_option(pool, key: str, value: int) -> None:
    _check(lib().slora_set_option(pool, key.encode(), value))
