"""The pins must notice a mistake anywhere in the oracle: each planted bug (in a compiled copy
of oracle/slora_oracle.c, on the CPU) has to fail at least one pin check."""
import ctypes as C
import os
import subprocess

import numpy as np
import pytest

from paper_2311_03285_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "slora_oracle.c")

MUTANTS = {
    "dropped y_in": ("yo[d] = (double)yi[d];", "yo[d] = 0.0;"),
    "delta subtracted": ("yo[d] += s;", "yo[d] -= s;"),
    "B list read from the A list": ("const int32_t *pb = pa + r;", "const int32_t *pb = pa;"),
    "last column of H skipped in the shrink": ("for (int32_t h = 0; h < H; ++h)\n                    s += widen(xt[h]",
                                               "for (int32_t h = 0; h < H - 1; ++h)\n                    s += widen(xt[h]"),
    "last rank skipped in the expand": ("for (int32_t j = 0; j < r; ++j)\n                    s += v[j]",
                                        "for (int32_t j = 0; j < r - 1; ++j)\n                    s += v[j]"),
    "first rank skipped in the shrink": ("for (int32_t j = 0; j < r; ++j) {\n                const uint16_t *acol",
                                         "for (int32_t j = 1; j < r; ++j) {\n                const uint16_t *acol"),
    "x of the wrong token": ("const uint16_t *xt = x + (int64_t)t * H;", "const uint16_t *xt = x + (int64_t)(t > 0 ? t - 1 : 0) * H;"),
    "page index off by one": ("const uint16_t *acol = pool + (int64_t)pa[j] * H;",
                              "const uint16_t *acol = pool + (int64_t)(pa[j] > 0 ? pa[j] - 1 : 0) * H;"),
    "B indexed by column then rank": ("widen(pool[(int64_t)pb[j] * H + d], dtype)", "widen(pool[(int64_t)pb[j] * H + (H - 1 - d)], dtype)"),
    "adapter of the previous token": ("int32_t i = ids[t];\n            if (i == -1)\n                continue;\n            int32_t r = rank[i];",
                                      "int32_t i = ids[t > 0 ? t - 1 : 0];\n            if (i == -1)\n                continue;\n            int32_t r = rank[i];"),
    "fp16 exponent bias off by one": ("m = ldexp((double)(f | 0x400), e - 25);", "m = ldexp((double)(f | 0x400), e - 24);"),
    "bf16 fraction width wrong": ("int f = b & 0x7f;", "int f = b & 0x3f;"),
    "v scaled by 1/r": ("v[j] = s;", "v[j] = s / r;"),
}


def _load(path):
    L = C.CDLL(path)
    L.slo_lora_apply.restype = C.c_int
    L.slo_lora_apply.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p,
                                 C.c_int32, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int,
                                 C.c_void_p]
    return L


def _apply(L, pool, dtype, lists, ids, x_bits, y_in):
    from oracle.c_oracle import pack_lists
    pool = np.ascontiguousarray(pool, np.uint16)
    ids = np.ascontiguousarray(ids, np.int32)
    T, H = ids.size, pool.shape[1]
    x = np.ascontiguousarray(x_bits, np.uint16).reshape(T, H)
    yi = np.ascontiguousarray(y_in, np.float32).reshape(T, H)
    n_ad = max(lists) + 1
    rank, off, pl = pack_lists(lists, n_ad)
    out = np.empty((T, H), np.float64)
    p = lambda a: C.c_void_p(a.ctypes.data)
    rc = L.slo_lora_apply(p(pool), pool.shape[0], H, dtype, p(rank), p(off), p(pl), n_ad, p(ids), T, p(x), p(yi),
                          p(out), 1, None)
    assert rc == 0
    return out


def _pins_hold(L):
    """A compact version of the pins: the hand-worked example plus dense materialisation in both
    storage types.  Returns True when every check passes."""
    def dec(bits, dtype):
        b = np.ascontiguousarray(bits, np.uint16)
        if dtype == synth.F16:
            return b.view(np.float16).astype(np.float64)
        return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)

    # hand-worked example (tests/golden/worked_example_eq2.txt)
    f16 = lambda a: np.asarray(a, np.float16).view(np.uint16)
    pool = np.full((8, 4), synth.nan_bits(synth.F16), np.uint16)
    for pg, v in {5: [1, 0, 2, 0], 2: [0, 1, 0, -1], 7: [1, 2, 3, 4], 0: [.5, 0, -.5, 1], 3: [2, 2, 2, 2],
                  6: [-1, 0, 1, .25]}.items():
        pool[pg] = f16(v)
    lists = {0: np.array([[5, 2], [7, 0]], np.int32), 1: np.array([[3], [6]], np.int32)}
    x = np.stack([f16([1, 2, 3, 4]), f16([1, -1, .5, 0]), f16([9, 9, 9, 9])])
    y = np.array([[10, 20, 30, 40], [0, 0, 0, 0], [1, 2, 3, 4]], np.float32)
    out = _apply(L, pool, synth.F16, lists, [0, 1, -1], x, y)
    if not np.array_equal(out, np.array([[16, 34, 52, 66], [-1, 0, 1, .25], [1, 2, 3, 4]], np.float64)):
        return False
    for dtype in (synth.F16, synth.BF16):
        g = np.random.default_rng(5)
        ids = g.integers(0, 4, size=9)
        w = synth.make_workload("m", 5, 64, dtype, 40, 1, (3, 0, 5, 1), ids)
        pool = w.dense_pool_bits()
        lists = {a: w.page_idx[a][0] for a in range(4)}
        out = _apply(L, pool, dtype, lists, w.ids, w.x_bits(), w.y_in())
        xx = dec(w.x_bits(), dtype)
        for t in range(w.T):
            i = int(w.ids[t])
            ref = w.y_in()[t].astype(np.float64)
            if w.ranks[i] > 0:
                ref = ref + xx[t] @ (dec(w.weight_bits(i, 0, 0), dtype).T @ dec(w.weight_bits(i, 0, 1), dtype))
            if not np.allclose(out[t], ref, rtol=1e-12, atol=1e-12):
                return False
    return True


def _build(text, path):
    src = path + ".c"
    open(src, "w").write(text)
    subprocess.check_call(["gcc", "-std=c11", "-O1", "-fPIC", "-shared", "-fopenmp", "-o", path, src, "-lm"])
    return _load(path)


def test_the_unmodified_oracle_passes_the_compact_pins(tmp_path):
    assert _pins_hold(_build(open(SRC).read(), str(tmp_path / "orig.so")))


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_each_planted_bug_is_caught(tmp_path, name):
    old, new = MUTANTS[name]
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation site for '{name}' not found exactly once"
    L = _build(text.replace(old, new), str(tmp_path / "mut.so"))
    assert not _pins_hold(L), f"no pin noticed: {name}"
