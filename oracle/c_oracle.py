"""ctypes front end of the C oracle (oracle/slora_oracle.c).  Test infrastructure only."""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional, Sequence, Tuple

import numpy as np

from . import build as _build

_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        path = _build.LIB if os.path.exists(_build.LIB) else _build.build()
        L = C.CDLL(path)
        L.slo_f16_to_f64.restype = C.c_double
        L.slo_f16_to_f64.argtypes = [C.c_uint16]
        L.slo_bf16_to_f64.restype = C.c_double
        L.slo_bf16_to_f64.argtypes = [C.c_uint16]
        L.slo_widen.restype = None
        L.slo_widen.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_void_p]
        L.slo_gather.restype = C.c_int
        L.slo_gather.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_int, C.c_void_p, C.c_int32, C.c_void_p]
        L.slo_gather_bits.restype = C.c_int
        L.slo_gather_bits.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_int32, C.c_void_p]
        L.slo_lora_apply.restype = C.c_int
        L.slo_lora_apply.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_int, C.c_void_p, C.c_void_p,
                                     C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p,
                                     C.c_void_p, C.c_void_p, C.c_int, C.c_void_p]
        L.slo_f64_to_16.restype = C.c_uint16
        L.slo_f64_to_16.argtypes = [C.c_double, C.c_int]
        L.slo_round16.restype = None
        L.slo_round16.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_void_p]
        _lib = L
    return _lib


def _p(a: np.ndarray) -> C.c_void_p:
    return C.c_void_p(a.ctypes.data)


def widen(bits: np.ndarray, dtype: int) -> np.ndarray:
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    out = np.empty(b.shape, dtype=np.float64)
    lib().slo_widen(_p(b), b.size, dtype, _p(out))
    return out


def gather(pool: np.ndarray, dtype: int, pages: Sequence[int]) -> np.ndarray:
    """fp64 [r, H]: row j = page pages[j] of the pool."""
    pool = np.ascontiguousarray(pool, dtype=np.uint16)
    pg = np.ascontiguousarray(pages, dtype=np.int32)
    n_pages, H = pool.shape
    out = np.empty((pg.size, H), dtype=np.float64)
    rc = lib().slo_gather(_p(pool), n_pages, H, dtype, _p(pg), pg.size, _p(out))
    if rc:
        raise IndexError("page index out of range")
    return out


def gather_bits(pool: np.ndarray, pages: Sequence[int]) -> np.ndarray:
    pool = np.ascontiguousarray(pool, dtype=np.uint16)
    pg = np.ascontiguousarray(pages, dtype=np.int32)
    n_pages, H = pool.shape
    out = np.empty((pg.size, H), dtype=np.uint16)
    rc = lib().slo_gather_bits(_p(pool), n_pages, H, _p(pg), pg.size, _p(out))
    if rc:
        raise IndexError("page index out of range")
    return out


def pack_lists(lists: Dict[int, np.ndarray], n_adapters: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """lists[a] = int32 [2, r] (A pages, B pages) -> (rank, list_off, flat page list)."""
    rank = np.zeros(n_adapters, dtype=np.int32)
    off = np.zeros(n_adapters, dtype=np.int64)
    flat, at = [], 0
    for a in range(n_adapters):
        if a in lists:
            l = np.ascontiguousarray(lists[a], dtype=np.int32)
            rank[a] = l.shape[1]
            off[a] = at
            flat.append(l.reshape(-1))
            at += l.size
    pl = np.concatenate(flat).astype(np.int32) if flat else np.zeros(1, dtype=np.int32)
    return rank, off, pl


def lora_apply(pool: np.ndarray, dtype: int, lists: Dict[int, np.ndarray], ids: np.ndarray,
               x_bits: np.ndarray, y_in: np.ndarray, n_threads: int = 0,
               return_threads: bool = False):
    """y_out (fp64 [T, H]) = y_in + per-token x A_i B_i for one slot.

    lists[a] = int32 [2, r_a]: pool rows holding A's columns, then B's rows.
    """
    pool = np.ascontiguousarray(pool, dtype=np.uint16)
    n_pages, H = pool.shape
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    T = ids.size
    x = np.ascontiguousarray(x_bits, dtype=np.uint16).reshape(T, H)
    yi = np.ascontiguousarray(y_in, dtype=np.float32).reshape(T, H)
    n_adapters = (max(lists) + 1) if lists else 0
    rank, off, pl = pack_lists(lists, n_adapters)
    out = np.empty((T, H), dtype=np.float64)
    used = C.c_int(0)
    rc = lib().slo_lora_apply(_p(pool), n_pages, H, dtype, _p(rank), _p(off), _p(pl), n_adapters,
                              _p(ids), T, _p(x), _p(yi), _p(out), n_threads, C.byref(used))
    if rc == -1:
        raise IndexError("page index out of range")
    if rc == -2:
        raise KeyError("adapter id out of range")
    if rc:
        raise MemoryError("oracle allocation failed")
    return (out, used.value) if return_threads else out


def round16(values: np.ndarray, dtype: int) -> np.ndarray:
    """fp64 -> bit patterns of the nearest binary16 / bfloat16 values (ties to even, one rounding)."""
    v = np.ascontiguousarray(values, dtype=np.float64)
    out = np.empty(v.shape, dtype=np.uint16)
    lib().slo_round16(_p(v), v.size, dtype, _p(out))
    return out


def lora_apply_y16(pool: np.ndarray, dtype: int, lists: Dict[int, np.ndarray], ids: np.ndarray,
                   x_bits: np.ndarray, y_bits: np.ndarray, n_threads: int = 0):
    """16-bit y: returns (bit patterns of the rounded result, the fp64 result before rounding).

    y_bits holds y_in in the pool's storage type; its values are exact in fp32.
    """
    y32 = widen(y_bits, dtype).astype(np.float32)
    exact = lora_apply(pool, dtype, lists, ids, x_bits, y32, n_threads)
    return round16(exact, dtype), exact
