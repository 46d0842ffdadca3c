"""Independent numpy fp64 formulation of the oracle.  Test infrastructure only.

Same definition as oracle/slora_oracle.c (Sec. 2 Eq. 2 evaluated per token with that token's
adapter, weights read through page lists as in Sec. 5.1) but written with numpy views for the
16-bit decoding and numpy matrix products for the two steps, so that a slip in the C loops
(index, orientation, dropped term) does not repeat here.
"""
from __future__ import annotations

from typing import Dict, Sequence

import numpy as np

F16, BF16 = 0, 1


def widen(bits: np.ndarray, dtype: int) -> np.ndarray:
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    if dtype == F16:
        return b.view(np.float16).astype(np.float64)
    if dtype == BF16:
        return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    raise ValueError(dtype)


def gather(pool: np.ndarray, dtype: int, pages: Sequence[int]) -> np.ndarray:
    pg = np.asarray(pages, dtype=np.int64)
    if pg.size and (pg.min() < 0 or pg.max() >= pool.shape[0]):
        raise IndexError("page index out of range")
    return widen(pool[pg], dtype)


def gather_bits(pool: np.ndarray, pages: Sequence[int]) -> np.ndarray:
    pg = np.asarray(pages, dtype=np.int64)
    if pg.size and (pg.min() < 0 or pg.max() >= pool.shape[0]):
        raise IndexError("page index out of range")
    return np.ascontiguousarray(pool[pg], dtype=np.uint16)


def lora_apply(pool: np.ndarray, dtype: int, lists: Dict[int, np.ndarray], ids: np.ndarray,
               x_bits: np.ndarray, y_in: np.ndarray) -> np.ndarray:
    ids = np.asarray(ids, dtype=np.int64)
    T = ids.size
    H = pool.shape[1]
    x = widen(np.asarray(x_bits).reshape(T, H), dtype)
    out = np.asarray(y_in, dtype=np.float32).reshape(T, H).astype(np.float64)
    for t in range(T):
        i = int(ids[t])
        if i == -1:
            continue
        if i not in lists:
            raise KeyError("adapter id out of range")
        pa, pb = lists[i]
        if len(pa) == 0:
            continue
        At = gather(pool, dtype, pa)          # [r, H]: row j = column j of A
        B = gather(pool, dtype, pb)           # [r, H]: row j = row j of B
        v = At @ x[t]                         # v[j] = sum_h x[h] A[h, j]
        out[t] = out[t] + v @ B
    return out
