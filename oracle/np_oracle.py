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


def round16(values: np.ndarray, dtype: int) -> np.ndarray:
    """fp64 -> bit patterns of the nearest 16-bit values, ties to even, rounded once.

    Integer formulation on the fp64 bit pattern (the C oracle scales with ldexp and rounds with
    nearbyint): the value is m * 2^(e-52) with a 53-bit integer m; dropping `sh` low bits with
    round-half-even gives the target significand, a carry out of it bumps the exponent.
    """
    p, emin, emax = (11, -14, 15) if dtype == F16 else (8, -126, 127)
    fbits = p - 1
    v = np.ascontiguousarray(values, dtype=np.float64)
    u = v.view(np.uint64).reshape(-1)
    sign = ((u >> np.uint64(63)) << np.uint64(15)).astype(np.uint32)
    ef = ((u >> np.uint64(52)) & np.uint64(0x7FF)).astype(np.int64)
    frac = (u & np.uint64((1 << 52) - 1)).astype(np.int64)
    out = np.zeros(u.shape, dtype=np.uint32)
    inf = np.uint32((2 * emax + 1) << fbits)
    special = ef == 0x7FF
    out[special & (frac == 0)] = inf
    out[special & (frac != 0)] = inf | np.uint32(1 << (fbits - 1))
    # fp64 subnormals are far below half the smallest 16-bit subnormal: they round to zero
    fin = (~special) & (ef != 0)
    e = ef[fin] - 1023                                  # unbiased exponent, value = m * 2^(e-52)
    m = frac[fin] | (1 << 52)
    et = np.maximum(e, emin)                            # exponent whose spacing applies
    sh = 52 - fbits + (et - e)                          # low bits to drop (>= 42)
    sh_c = np.minimum(sh, 62)
    m = np.where(sh > 62, 0, m)                         # far below half a unit: rounds to zero
    q = m >> sh_c
    rem = m & ((np.int64(1) << sh_c) - 1)
    half = np.int64(1) << (sh_c - 1)
    q = q + ((rem > half) | ((rem == half) & ((q & 1) == 1)))
    carry = q >= (1 << p)
    q = np.where(carry, 1 << fbits, q)
    et = et + carry
    bits = np.where(q < (1 << fbits), q, ((et + emax) << fbits) | (q - (1 << fbits)))
    bits = np.where(et > emax, int(inf), bits)
    out[fin] = bits.astype(np.uint32)
    return (out | sign).astype(np.uint16).reshape(v.shape)


def lora_apply_y16(pool, dtype, lists, ids, x_bits, y_bits):
    exact = lora_apply(pool, dtype, lists, ids, x_bits, widen(y_bits, dtype).astype(np.float32))
    return round16(exact, dtype), exact
