"""GPU parity of the 16-bit-y variant (y in the pool's storage type, rounded once at the store).

The oracle rounds the exact fp64 result once to the 16-bit type; the kernels round their fp32
sum, whose accumulation error is a few 1e-7 of the size of the terms.  The bar, per element:
  * |gpu - exact| <= half the spacing of the 16-bit format at the GPU's value
                     + 4e-6 * max(1, |exact|, |y_in|)
    i.e. a correctly rounded result up to the fp32 accumulation slack (where y_in and the delta
    cancel, that slack is several units in the last place of the small result);
  * at most 1 % of the elements differ from the oracle's own rounding at all.
Integer-valued inputs have exact fp32 sums: there the bits must be equal everywhere.
Rows with no adapter or a rank-0 adapter keep their bits.
"""
import numpy as np
import pytest
import torch

from oracle import c_oracle
from paper_2311_03285_amd import slora, synth
from paper_2311_03285_amd.harness import DeviceWorkload, bits_to_device
from test_gpu_mfma import MFMA_ALL, VEC_ONLY, prefill_workload, route
from test_gpu_parity import ragged_workload

pytestmark = pytest.mark.gpu


def dec(bits, dtype):
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    if dtype == synth.F16:
        return b.view(np.float16).astype(np.float64)
    return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def oracle_y16(w, slot, y_bits=None, x_bits=None):
    used = np.unique(w.ids[w.ids >= 0])
    rows, lists = w.compact_pool(slot, used)
    if rows.shape[0] == 0:
        rows = np.zeros((1, w.H), dtype=np.uint16)
    return c_oracle.lora_apply_y16(rows, w.dtype, lists, w.ids, w.x_bits(slot) if x_bits is None else x_bits,
                                   w.y16_bits(slot) if y_bits is None else y_bits)


def gpu_y16(dw, slots, plan=None, y_bits=None):
    w = dw.w
    plan = dw.plan() if plan is None else plan
    xs = [dw.x_dev(s) for s in slots]
    ys = [bits_to_device(w.y16_bits(s) if y_bits is None else y_bits, dw.device) for s in slots]
    slora.lora_apply_multi_y16(plan, slots, [t.data_ptr() for t in xs], [t.data_ptr() for t in ys])
    torch.cuda.synchronize(dw.device)
    return [t.cpu().numpy().view(np.uint16).reshape(w.T, w.H) for t in ys]


def assert_y16_close(got_bits, ref_bits, exact, y_in_bits, dtype, what=""):
    got = dec(got_bits, dtype)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    frac = float(np.mean(got_bits != ref_bits))
    assert frac <= 0.01, f"{what}: {frac:.4f} of the elements differ from the oracle's rounding"
    mag = (got_bits & 0x7FFF).astype(np.uint16)
    spacing = dec(mag + np.uint16(1), dtype) - dec(mag, dtype)      # to the next 16-bit value up
    slack = 4e-6 * np.maximum(1.0, np.maximum(np.abs(exact), np.abs(dec(y_in_bits, dtype))))
    err = np.abs(got - exact)
    worst = float(np.max(err - 0.5 * spacing - slack))
    assert worst <= 0.0, f"{what}: an element is {worst:.3e} beyond half a unit in the last place + slack"
    return frac


@pytest.mark.parametrize("n", [1, 2])
def test_configs_1_and_2_decode(n):
    w = synth.config(n)
    with DeviceWorkload(w, real_adapters="all") as dw:
        got = gpu_y16(dw, [0])[0]
        ref, exact = oracle_y16(w, 0)
        assert_y16_close(got, ref, exact, w.y16_bits(0), w.dtype, f"cfg{n}")


@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
@pytest.mark.parametrize("path", ["vec", "mfma"])
def test_ragged_shapes_on_both_kernel_families(dtype, path):
    w = prefill_workload(700, dtype, H=1000) if path == "mfma" else ragged_workload(701, dtype, H=1000)
    with DeviceWorkload(w, real_adapters="all", max_rank=160) as dw:
        route(dw.pool, MFMA_ALL if path == "mfma" else VEC_ONLY)
        plan = dw.plan()
        info = slora.plan_info(plan)
        assert (info["groups_vec"] == 0) == (path == "mfma")
        got = gpu_y16(dw, [0, 1], plan)
        for slot in (0, 1):
            ref, exact = oracle_y16(w, slot)
            assert_y16_close(got[slot], ref, exact, w.y16_bits(slot), dtype, f"{path} slot {slot}")
            quiet = (w.ids < 0) | (w.ranks[np.maximum(w.ids, 0)] == 0)
            assert quiet.any() and np.array_equal(got[slot][quiet], w.y16_bits(slot)[quiet])
        # one slot on its own, and a second run, give the same bits
        assert np.array_equal(gpu_y16(dw, [1], plan)[0], got[1])
        assert np.array_equal(gpu_y16(dw, [0, 1], plan)[0], got[0])


@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
@pytest.mark.parametrize("path", ["vec", "mfma", "split"])
def test_integer_valued_inputs_are_bit_exact(dtype, path):
    if path == "mfma":
        w = prefill_workload(710, dtype, H=512, int_valued=True)
    else:
        w = ragged_workload(711, dtype, H=512 if path == "split" else 1536, int_valued=True)
    with DeviceWorkload(w, real_adapters="all", max_rank=160) as dw:
        route(dw.pool, MFMA_ALL if path == "mfma" else VEC_ONLY)
        got = gpu_y16(dw, [0])[0]
        ref, exact = oracle_y16(w, 0)
        assert np.array_equal(got, ref)


def test_zero_B_leaves_y_unchanged():
    w = ragged_workload(720, synth.BF16, H=1000)
    with DeviceWorkload(w, real_adapters="all") as dw:
        pages = np.concatenate([w.page_idx[a][0, 1] for a in range(w.n_adapters)])
        slora.pool_write_pages(dw.pool, pages, np.zeros((pages.size, w.H), np.uint16), False)
        yb = w.y16_bits(0).copy()
        yb[yb == 0x8000] = 0                       # -0 + 0 = +0 would change the sign bit
        got = gpu_y16(dw, [0], y_bits=yb)[0]
        assert np.array_equal(got, yb)


def test_expand_stage_on_its_own_and_argument_errors():
    w = ragged_workload(730, synth.F16, H=1000)
    with DeviceWorkload(w, real_adapters="all") as dw:
        plan = dw.plan()
        want = gpu_y16(dw, [0, 1], plan)
        xs = [dw.x_dev(s) for s in (0, 1)]
        ys = [bits_to_device(w.y16_bits(s), dw.device) for s in (0, 1)]
        slora.lora_shrink(plan, [0, 1], [t.data_ptr() for t in xs])
        slora.lora_expand_y16(plan, [0, 1], [t.data_ptr() for t in ys])
        torch.cuda.synchronize()
        for s in (0, 1):
            assert np.array_equal(ys[s].cpu().numpy().view(np.uint16).reshape(w.T, w.H), want[s])
        before = ys[0].clone()
        with pytest.raises(slora.SloraError):     # the same buffer twice
            slora.lora_apply_multi_y16(plan, [0, 1], [t.data_ptr() for t in xs], [ys[0].data_ptr()] * 2)
        with pytest.raises(slora.SloraError):     # misaligned y
            slora.lora_apply_multi_y16(plan, [0], [xs[0].data_ptr()], [ys[0].data_ptr() + 2])
        torch.cuda.synchronize()
        assert torch.equal(before, ys[0])          # a rejected call touches nothing


def test_config3_prefill_full_size_y16():
    """Full size, in the multi-slot launch shape the bench times."""
    w = synth.config(3)
    slots = [0, 3]
    with DeviceWorkload(w, real_adapters="used", slots=slots) as dw:
        got = gpu_y16(dw, slots)
        for k, slot in enumerate(slots):
            ref, exact = oracle_y16(w, slot)
            assert_y16_close(got[k], ref, exact, w.y16_bits(slot), w.dtype, f"cfg3 slot {slot}")


def test_config4_decode_full_size_y16():
    w = synth.config(4)
    slots = [0, 1, 2, 3]
    with DeviceWorkload(w, real_adapters="used", slots=slots) as dw:
        got = gpu_y16(dw, slots)
        for k, slot in enumerate(slots):
            ref, exact = oracle_y16(w, slot)
            assert_y16_close(got[k], ref, exact, w.y16_bits(slot), w.dtype, f"cfg4 slot {slot}")


def test_config5_mixed_full_size_y16():
    """bfloat16, prefill requests and decode tokens in one batch: both kernel families in one call."""
    w = synth.config(5)
    slots = [0, 15]
    with DeviceWorkload(w, real_adapters="used", slots=slots) as dw:
        got = gpu_y16(dw, slots)
        for k, slot in enumerate(slots):
            ref, exact = oracle_y16(w, slot)
            assert_y16_close(got[k], ref, exact, w.y16_bits(slot), w.dtype, f"cfg5 slot {slot}")


@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
@pytest.mark.parametrize("T", [3, 40])                 # vector kernels / MFMA kernels
def test_ties_round_to_even_on_the_device(dtype, T):
    """x = e_0 and A's only column = e_0 give v = 1 exactly, so the delta is B's row: with y_in on a
    16-bit grid point and B at half a spacing (and just beside it) the fp32 sum is exact and the
    store must round it as IEEE 754 roundTiesToEven does - even neighbour on ties."""
    H, dev = 64, torch.device("cuda:0")
    p = 11 if dtype == synth.F16 else 8
    half = 2.0 ** -p                                   # half the spacing of the format in [1, 2)
    enc = (lambda a: np.asarray(a, np.float16).view(np.uint16)) if dtype == synth.F16 else \
          (lambda a: (np.asarray(a, np.float32).view(np.uint32) >> 16).astype(np.uint16))
    even, odd = 1.0, 1.0 + 2 * half                    # last significand bit 0 / 1
    y_vals = np.tile([even, odd, -even, -odd, even, odd, even, odd], H // 8)
    b_vals = np.tile([half, half, -half, -half, 1.5 * half, 1.5 * half, 0.5 * half, 0.5 * half], H // 8)
    for v in (y_vals, b_vals):                         # all exactly representable in the 16-bit type
        assert np.array_equal(c_oracle.widen(enc(v), dtype), v)
    pool_bits = np.zeros((4, H), np.uint16)
    e0 = np.zeros(H)
    e0[0] = 1.0
    pool_bits[2] = enc(e0)                             # A: its one column
    pool_bits[1] = enc(b_vals)                         # B: its one row
    pool_t = torch.from_numpy(pool_bits.view(np.int16)).to(dev)
    pool = slora.pool_init(H, 4, dtype, pool_t.data_ptr(), 1, 1)
    slora.adapter_load(pool, 0, 1, [2, 1])
    slora.set_option(pool, "mfma_min_tiles", 1)
    ids = np.zeros(T, np.int32)
    x = bits_to_device(np.tile(enc(e0), (T, 1)), dev)
    yb = np.tile(enc(y_vals), (T, 1))
    y = bits_to_device(yb, dev)
    plan = slora.batch_plan(pool, ids, None)
    assert (slora.plan_info(plan)["groups_mfma"] == 1) == (T >= 16)
    slora.lora_apply_multi_y16(plan, [0], [x.data_ptr()], [y.data_ptr()])
    torch.cuda.synchronize()
    got = y.cpu().numpy().view(np.uint16)
    ref, exact = c_oracle.lora_apply_y16(pool_bits, dtype, {0: np.array([[2], [1]], np.int32)}, ids,
                                         np.tile(enc(e0), (T, 1)), yb)
    assert np.array_equal(exact[T - 1], y_vals + b_vals)
    # ties go to the even neighbour: 1 + h -> 1, (1 + 2h) + h -> 1 + 4h; 1.5 h rounds up, 0.5 h down
    want = np.tile([even, odd + 2 * half, -even, -(odd + 2 * half), even + 2 * half, odd + 2 * half, even, odd], H // 8)
    assert np.array_equal(ref[T - 1], enc(want))
    assert np.array_equal(got, ref)
    slora.plan_destroy(plan)
    slora.pool_destroy(pool)


@pytest.mark.parametrize("path", ["vec", "mfma"])
def test_extreme_shapes_y16(path):
    """The largest page (H = 32768) and the largest rank (1024) with 16-bit y."""
    cases = [
        synth.make_workload("max-H", 905, 32768, synth.BF16, 128, 1, (8, 40),
                            np.array([0, 1, 1, 0, 1, -1, 1, 1], dtype=np.int32)),
        synth.make_workload("max-rank", 906, 256, synth.F16, 4200, 1, (1024, 1000),
                            np.repeat([0, 1], [3, 40]).astype(np.int32), np.array([0, 3, 43], dtype=np.int32)),
    ]
    for w in cases:
        with DeviceWorkload(w, real_adapters="all", max_rank=1024) as dw:
            slora.set_option(dw.pool, "mfma_min_tokens", VEC_ONLY if path == "vec" else 1)
            slora.set_option(dw.pool, "mfma_min_tiles", 1)
            got = gpu_y16(dw, [0])[0]
            ref, exact = oracle_y16(w, 0)
            assert_y16_close(got, ref, exact, w.y16_bits(0), w.dtype, f"{w.name} {path}")
