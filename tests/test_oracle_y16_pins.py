"""Pins for the oracle's 16-bit-output leg: the final rounding of y to binary16 / bfloat16.

The rounding is fixed to things other than itself: numpy's correctly rounded float64 -> float16
conversion, the textbook add-and-shift rounding of a float32 pattern to bfloat16 (on inputs that
are exact in float32, so no second rounding is involved), and the definition of
round-to-nearest-even checked on every pair of neighbouring 16-bit values (a value survives a
round trip; the midpoint goes to the even neighbour; one fp64 step either side of the midpoint
goes to the nearer neighbour; overflow and gradual underflow at the ends of the range).
The composed result (y_in + xAB, rounded once) is pinned by one-hot closed forms computed with
numpy float16 arithmetic and by the exact-zero cases.
"""
import ctypes as C
import os
import subprocess

import numpy as np
import pytest

from paper_2311_03285_amd import synth

IMPLS = ["c", "np"]
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "slora_oracle.c")


def dec(bits, dtype):
    """16-bit patterns -> float64 by library views only."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    if dtype == synth.F16:
        return b.view(np.float16).astype(np.float64)
    return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def finite_positive_patterns(dtype):
    top = 0x7C00 if dtype == synth.F16 else 0x7F80      # +inf
    return np.arange(0, top, dtype=np.uint16)


def neighbour_checks(round16, dtype):
    """True when round16 behaves as round-to-nearest-even on every neighbouring pair."""
    lo = finite_positive_patterns(dtype)
    hi = (lo + 1).astype(np.uint16)                     # last one is +inf
    a, b = dec(lo, dtype), dec(hi, dtype)
    finite = np.isfinite(b)
    # the value just above the largest finite one behaves as if the format went on: 2^(emax+1)
    b_ext = np.where(finite, b, 2.0 * dec(np.array([0x7BFF if dtype == synth.F16 else 0x7F7F], np.uint16), dtype)[0]
                     - a[-2])
    mid = 0.5 * (a + b_ext)                             # exact: both have at most 12 significant bits
    even = np.where(lo % 2 == 0, lo, hi)
    ok = True
    for sgn, sbit in ((1.0, 0), (-1.0, 0x8000)):
        ok &= np.array_equal(round16(sgn * a, dtype), lo | sbit)                          # round trip
        ok &= np.array_equal(round16(sgn * mid, dtype), even | sbit)                      # tie -> even
        ok &= np.array_equal(round16(sgn * np.nextafter(mid, np.inf), dtype), hi | sbit)  # above the tie
        ok &= np.array_equal(round16(sgn * np.nextafter(mid, 0.0), dtype), lo | sbit)     # below the tie
    return bool(ok)


def get_round16(oracles, impl):
    return oracles[impl].round16


# ------------------------------------------------------------------ the rounding itself
@pytest.mark.parametrize("impl", IMPLS)
@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
def test_every_neighbouring_pair_rounds_to_nearest_even(oracles, impl, dtype):
    assert neighbour_checks(get_round16(oracles, impl), dtype)


@pytest.mark.parametrize("impl", IMPLS)
def test_binary16_rounding_equals_numpy_conversion(oracles, impl):
    g = np.random.default_rng(7)
    v = g.standard_normal(400_000) * g.choice([1e-9, 6e-8, 1e-6, 1e-4, 1.0, 100.0, 3e4, 7e4, 1e39], 400_000)
    v = np.concatenate([v, [0.0, -0.0, np.inf, -np.inf, 65504.0, 65519.99, 65520.0, 2.0**-24, 2.0**-25,
                            np.nextafter(2.0**-25, 1.0), 3 * 2.0**-25]])
    with np.errstate(over="ignore"):
        ref = v.astype(np.float16).view(np.uint16)
    assert np.array_equal(get_round16(oracles, impl)(v, synth.F16), ref)


@pytest.mark.parametrize("impl", IMPLS)
def test_bfloat16_rounding_equals_add_and_shift_on_float32_inputs(oracles, impl):
    g = np.random.default_rng(8)
    with np.errstate(over="ignore"):
        f = (g.standard_normal(400_000) * g.choice([1e-38, 1e-30, 1e-3, 1.0, 1e5, 1e30, 3e38], 400_000)).astype(np.float32)
    f = f[np.isfinite(f)]
    u = f.view(np.uint32).astype(np.uint64)
    ref = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)      # overflow lands on the inf pattern
    assert np.array_equal(get_round16(oracles, impl)(f.astype(np.float64), synth.BF16), ref)


@pytest.mark.parametrize("impl", IMPLS)
@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
def test_special_values(oracles, impl, dtype):
    r = get_round16(oracles, impl)
    inf = 0x7C00 if dtype == synth.F16 else 0x7F80
    out = r(np.array([0.0, -0.0, np.inf, -np.inf, 1e300, -1e300, 1e-300, -1e-300, 5e-324]), dtype)
    assert list(out) == [0, 0x8000, inf, 0x8000 | inf, inf, 0x8000 | inf, 0, 0x8000, 0]
    nan = int(r(np.array([np.nan]), dtype)[0])
    assert (nan & inf) == inf and (nan & (inf ^ 0x7FFF)) != 0           # exponent all ones, fraction non-zero


def test_c_and_numpy_roundings_agree(oracles):
    g = np.random.default_rng(9)
    v = g.standard_normal(300_000) * np.exp(g.uniform(-100, 100, 300_000))
    for dtype in (synth.F16, synth.BF16):
        assert np.array_equal(oracles["c"].round16(v, dtype), oracles["np"].round16(v, dtype))


# ------------------------------------------------------------------ planted bugs in the rounding
ROUND_MUTANTS = {
    "truncation instead of rounding": ("double n = nearbyint(ldexp(a, fbits - e));", "double n = floor(ldexp(a, fbits - e));"),
    "ties away from zero": ("double n = nearbyint(ldexp(a, fbits - e));", "double n = round(ldexp(a, fbits - e));"),
    "no gradual underflow": ("    if (e < emin)\n        e = emin; ", "    if (0)\n        e = emin; "),
    "carry into the next binade dropped": ("        e += 1;\n    }\n    if (e > emax)", "    }\n    if (e > emax)"),
    "bfloat16 keeps 7 significand bits": ("const int p = dtype == SLO_F16 ? 11 : 8; ", "const int p = dtype == SLO_F16 ? 11 : 7; "),
    "overflow saturates instead of going to infinity": ("    if (e > emax)\n        return (uint16_t)(sign | inf);",
                                                        "    if (e > emax)\n        return (uint16_t)(sign | (inf - 1));"),
}


def _round16_of(path):
    L = C.CDLL(path)
    L.slo_round16.restype = None
    L.slo_round16.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_void_p]

    def round16(v, dtype):
        v = np.ascontiguousarray(v, np.float64)
        out = np.empty(v.shape, np.uint16)
        L.slo_round16(C.c_void_p(v.ctypes.data), v.size, dtype, C.c_void_p(out.ctypes.data))
        return out
    return round16


def _build(text, path):
    open(path + ".c", "w").write(text)
    subprocess.check_call(["gcc", "-std=c11", "-O1", "-fPIC", "-shared", "-fopenmp", "-o", path, path + ".c", "-lm"])
    return _round16_of(path)


@pytest.mark.parametrize("name", sorted(ROUND_MUTANTS))
def test_each_planted_rounding_bug_is_caught(tmp_path, name):
    old, new = ROUND_MUTANTS[name]
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation site for '{name}' not found exactly once"
    assert neighbour_checks(_build(text, str(tmp_path / "orig.so")), synth.F16)
    r = _build(text.replace(old, new), str(tmp_path / "mut.so"))
    assert not (neighbour_checks(r, synth.F16) and neighbour_checks(r, synth.BF16)), f"no pin noticed: {name}"


# ------------------------------------------------------------------ the composed result
def _case(seed, dtype, H=64, ranks=(3, 0, 5, 1), T=9):
    g = np.random.default_rng(seed)
    ids = g.integers(0, len(ranks), size=T)
    ids[g.integers(0, T)] = -1
    w = synth.make_workload("y16", seed, H, dtype, 40, 1, ranks, ids)
    lists = {a: w.page_idx[a][0] for a in range(len(ranks))}
    return w, w.dense_pool_bits(), lists


@pytest.mark.parametrize("impl", IMPLS)
@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
def test_rows_without_a_delta_keep_their_bits(oracles, impl, dtype):
    w, pool, lists = _case(21, dtype)
    yb = w.y16_bits()
    bits, exact = oracles[impl].lora_apply_y16(pool, dtype, lists, w.ids, w.x_bits(), yb)
    quiet = (w.ids == -1) | (w.ranks[np.maximum(w.ids, 0)] == 0)
    assert quiet.any() and (~quiet).any()
    assert np.array_equal(bits[quiet], yb[quiet])
    assert not np.array_equal(bits[~quiet], yb[~quiet])
    # the rounded result is the nearest 16-bit value to the unrounded one: no neighbour is closer
    got = dec(bits, dtype)
    for step in (-1, 1):
        other = dec((bits.astype(np.int32) + step).astype(np.uint16), dtype)
        closer = np.abs(other - exact) < np.abs(got - exact)
        assert not np.any(closer & np.isfinite(other) & (np.sign(other) == np.sign(got)))


@pytest.mark.parametrize("impl", IMPLS)
def test_one_hot_inputs_reduce_to_one_float16_addition(oracles, impl):
    """x = e_h and A's pages one-hot: the delta is a row of B, so y_out = fl16(y_in + B[j, :]),
    which numpy's float16 addition (exact sum, rounded once) gives directly."""
    dtype, H = synth.F16, 64
    g = np.random.default_rng(3)
    B = g.standard_normal((2, H)).astype(np.float16)
    yin = g.standard_normal((2, H)).astype(np.float16)
    pool = np.zeros((8, H), np.uint16)
    A = np.zeros((2, H), np.float16)
    A[0, 5] = 1.0                                       # column 0 of A = e_5, column 1 = e_9
    A[1, 9] = 1.0
    pool[1], pool[6] = A.view(np.uint16)
    pool[3], pool[4] = B.view(np.uint16)
    lists = {0: np.array([[1, 6], [3, 4]], np.int32)}
    x = np.zeros((2, H), np.float16)
    x[0, 5] = 1.0                                       # token 0 picks B row 0
    x[1, 9] = 1.0                                       # token 1 picks B row 1
    bits, exact = oracles[impl].lora_apply_y16(pool, dtype, lists, np.array([0, 0]), x.view(np.uint16),
                                               yin.view(np.uint16))
    ref = (yin + B).view(np.uint16)                     # IEEE: the exact sum rounded once to binary16
    assert np.array_equal(bits, ref)
    assert np.array_equal(exact, yin.astype(np.float64) + B.astype(np.float64))


@pytest.mark.parametrize("impl", IMPLS)
@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
def test_y16_is_the_fp32_y_result_rounded_once(oracles, impl, dtype):
    """The 16-bit leg adds nothing but the final rounding to the pinned fp32-y oracle."""
    w, pool, lists = _case(22, dtype)
    yb = w.y16_bits()
    bits, exact = oracles[impl].lora_apply_y16(pool, dtype, lists, w.ids, w.x_bits(), yb)
    y32 = dec(yb, dtype).astype(np.float32)
    assert np.array_equal(exact, oracles[impl].lora_apply(pool, dtype, lists, w.ids, w.x_bits(), y32))
    if dtype == synth.F16:
        assert np.array_equal(bits, exact.astype(np.float16).view(np.uint16))


def test_c_and_numpy_y16_agree(oracles):
    for dtype in (synth.F16, synth.BF16):
        w, pool, lists = _case(23, dtype)
        a, ea = oracles["c"].lora_apply_y16(pool, dtype, lists, w.ids, w.x_bits(), w.y16_bits())
        b, eb = oracles["np"].lora_apply_y16(pool, dtype, lists, w.ids, w.x_bits(), w.y16_bits())
        assert np.allclose(ea, eb, rtol=1e-12, atol=1e-12)
        assert np.mean(a != b) < 0.01 and np.all(np.abs(a.astype(np.int32) - b.astype(np.int32)) <= 1)
