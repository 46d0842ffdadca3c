"""GPU parity of the MFMA (prefill) kernels and of the full-size configurations.

Same tolerance as the decode tests: rel-L2 <= 1e-3 and max-abs <= 1e-2 against the fp64
oracle; integer-valued inputs bit for bit.  The same batch is also forced through each of the
two kernel families, which must both stay inside the tolerance.
"""
import numpy as np
import pytest
import torch

from paper_2311_03285_amd import slora, synth
from paper_2311_03285_amd.harness import DeviceWorkload
from gpu_util import REL_L2_EXPECTED, assert_close, errors, gpu_slot, oracle_slot

pytestmark = pytest.mark.gpu

VEC_ONLY = 1 << 40
MFMA_ALL = 1


def route(pool, min_tokens, min_tiles=1):
    """Choose the kernel family: groups of >= min_tokens tokens go to the MFMA kernels, provided
    the batch has >= min_tiles 32-token tiles of them (1: no such condition)."""
    slora.set_option(pool, "mfma_min_tokens", min_tokens)
    slora.set_option(pool, "mfma_min_tiles", min_tiles)


def prefill_workload(seed, dtype, H=1000, ranks=(1, 3, 0, 5, 17, 8, 64, 33, 128, 160), lens=(1, 2, 31, 32, 33, 64, 65, 100, 7, 130),
                     n_slots=2, n_pages=1800, **kw):
    """Segments of ragged lengths around the tile sizes (32 / 64 tokens), odd ranks, one rank
    above 128 (two shrink rank chunks), a rank-0 adapter, and a few tokens without adapter."""
    g = np.random.default_rng(seed)
    seg = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    seg_ad = g.permutation(len(ranks))[:len(lens)]
    ids = np.repeat(seg_ad, lens).astype(np.int32)
    ids[seg[2]:seg[2] + 31] = -1                       # a whole segment without adapter
    return synth.make_workload("prefill-ragged", seed, H, dtype, n_pages, n_slots, ranks, ids, seg, **kw)


@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
@pytest.mark.parametrize("H", [64, 1000, 4096])
def test_forced_mfma_path(dtype, H):
    w = prefill_workload(400 + H, dtype, H=H)
    with DeviceWorkload(w, real_adapters="all", max_rank=160) as dw:
        route(dw.pool, MFMA_ALL)
        plan = dw.plan()
        info = slora.plan_info(plan)
        assert info["groups_vec"] == 0 and info["groups_mfma"] > 0
        for slot in range(w.n_slots):
            got = gpu_slot(dw, slot, plan)
            ref = oracle_slot(w, slot)
            rel, mx = assert_close(got, ref, f"mfma H={H} slot={slot}")
            assert rel <= 5e-6, rel
            untouched = (w.ids < 0) | (w.ranks[np.maximum(w.ids, 0)] == 0)
            assert np.array_equal(got[untouched], w.y_in(slot)[untouched])


@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
def test_both_paths_agree_with_the_oracle_on_the_same_batch(dtype):
    w = prefill_workload(450, dtype, H=512, y_zero=True)
    ref = oracle_slot(w, 0)
    outs = {}
    with DeviceWorkload(w, real_adapters="all", max_rank=160) as dw:
        for name, thr in (("vec", VEC_ONLY), ("mfma", MFMA_ALL), ("mixed", 16)):
            route(dw.pool, thr)
            outs[name] = gpu_slot(dw, 0, dw.plan())
            assert_close(outs[name], ref, name)
    rel, _ = errors(outs["vec"], outs["mfma"].astype(np.float64))
    assert rel <= 1e-5


@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
def test_mfma_integer_inputs_are_bit_exact(dtype):
    """Integer inputs: every product and partial sum is an integer below 2^22, so the 16-bit
    pieces of v, the MFMA products and the fp32 accumulation are all exact."""
    w = prefill_workload(460, dtype, H=512, int_valued=True)
    with DeviceWorkload(w, real_adapters="all", max_rank=160) as dw:
        route(dw.pool, MFMA_ALL)
        for slot in range(w.n_slots):
            got = gpu_slot(dw, slot)
            assert np.array_equal(got.astype(np.float64), oracle_slot(w, slot))


def test_mfma_zero_B_and_determinism():
    w = prefill_workload(470, synth.F16, H=512)
    with DeviceWorkload(w, real_adapters="all", max_rank=160) as dw:
        route(dw.pool, MFMA_ALL)
        plan = dw.plan()
        a = gpu_slot(dw, 1, plan)
        assert np.array_equal(a, gpu_slot(dw, 1, plan))
        pages = np.concatenate([w.page_idx[k][0, 1] for k in range(w.n_adapters)])
        slora.pool_write_pages(dw.pool, pages, np.zeros((pages.size, w.H), np.uint16), False)
        yi = w.y_in(0)
        yi[yi == 0] = 0.0
        got = gpu_slot(dw, 0, plan, y_in=yi)
        assert np.array_equal(got.view(np.uint32), yi.view(np.uint32))


def test_mfma_multi_slot_matches_single_slot():
    w = prefill_workload(480, synth.BF16, H=1000)
    with DeviceWorkload(w, real_adapters="all", max_rank=160) as dw:
        route(dw.pool, 16)                                   # both families
        plan = dw.plan()
        info = slora.plan_info(plan)
        assert info["groups_vec"] > 0 and info["groups_mfma"] > 0
        singles = [gpu_slot(dw, s, plan) for s in range(2)]
        xs = [dw.x_dev(0), dw.x_dev(1)]
        ys = [dw.y_dev(0), dw.y_dev(1)]
        slora.lora_apply_multi(plan, [0, 1], [t.data_ptr() for t in xs], [t.data_ptr() for t in ys])
        torch.cuda.synchronize()
        for s in range(2):
            assert np.array_equal(ys[s].cpu().numpy(), singles[s])


# ------------------------------------------------------------------ full-size configurations
def _full_config(n, slots, law="power"):
    """Full-size configuration in the launch shape the bench times: all checked slots in one
    multi-slot call (one launch pair), each slot against the oracle."""
    w = synth.config(n, law=law)
    with DeviceWorkload(w, real_adapters="used", slots=slots) as dw:
        plan = dw.plan()
        info = slora.plan_info(plan)
        xs = [dw.x_dev(s) for s in slots]
        ys = [dw.y_dev(s) for s in slots]
        slora.lora_apply_multi(plan, slots, [t.data_ptr() for t in xs], [t.data_ptr() for t in ys])
        torch.cuda.synchronize()
        for k, slot in enumerate(slots):
            got = ys[k].cpu().numpy()
            ref = oracle_slot(w, slot)
            rel, mx = assert_close(got, ref, f"cfg{n} slot {slot}")
            assert rel <= 5e-6, rel
            if k == 0:      # the single-slot call gives the same bits
                assert np.array_equal(got, gpu_slot(dw, slot, plan))
        # one adapter's pages, gathered back bit for bit from the scattered pool
        a = int(w.used_adapters()[0])
        assert np.array_equal(dw.gather(a, slots[0], 1), w.weight_bits(a, slots[0], 1))
    return info


def test_config3_prefill_full_size():
    info = _full_config(3, [0, 3])
    assert info["groups_mfma"] == info["groups"]            # every request is long enough for MFMA


@pytest.mark.parametrize("law", ["power", "zipf"])
def test_config4_large_pool_decode_full_size(law):
    """115 GB pool (byte offsets beyond 2^32), 2000 adapters, everything else marked KV."""
    info = _full_config(4, [0, 1, 2, 3], law)
    assert info["tokens"] == 256


def test_config5_mixed_full_size():
    info = _full_config(5, [0, 15])
    assert info["groups_mfma"] >= 8 and info["groups_vec"] > 100


def test_xcd_grouping_changes_the_schedule_not_the_result():
    w = prefill_workload(490, synth.F16, H=1000)
    with DeviceWorkload(w, real_adapters="all", max_rank=160) as dw:
        route(dw.pool, MFMA_ALL)
        slora.set_option(dw.pool, "xcd_group", 0)       # both lists round-robin over the dies
        a = gpu_slot(dw, 0, dw.plan())
        for mode in (1, 2, 3):                          # shrink list grouped, expand list, both
            slora.set_option(dw.pool, "xcd_group", mode)
            p = dw.plan()
            assert slora.plan_info(p)["mfma_shrink_items"] == slora.plan_info(dw.plans[0])["mfma_shrink_items"]
            assert np.array_equal(a, gpu_slot(dw, 0, p)), mode


def test_eight_slots_in_one_launch_pair():
    """The largest launch shape (8 slots per call, as the mixed configuration is timed): every
    slot gives the bits of that slot applied on its own, on a batch that uses both kernel
    families; with 16-bit y as well."""
    w = prefill_workload(495, synth.BF16, H=512, n_slots=8, n_pages=9000)
    with DeviceWorkload(w, real_adapters="all", max_rank=160) as dw:
        route(dw.pool, 16)                     # groups of >= 16 tokens on MFMA, the rest on the vector kernels
        plan = dw.plan()
        info = slora.plan_info(plan)
        assert info["groups_mfma"] > 0 and info["groups_vec"] > 0
        slots = list(range(8))
        single = [gpu_slot(dw, s, plan) for s in slots]
        xs = [dw.x_dev(s) for s in slots]
        ys = [dw.y_dev(s) for s in slots]
        slora.lora_apply_multi(plan, slots, [t.data_ptr() for t in xs], [t.data_ptr() for t in ys])
        torch.cuda.synchronize()
        for s in slots:
            assert np.array_equal(ys[s].cpu().numpy(), single[s]), s
        assert_close(single[7], oracle_slot(w, 7), "slot 7 of 8")
        # 16-bit y: eight slots at once against one at a time
        from paper_2311_03285_amd.harness import bits_to_device
        y16 = [bits_to_device(w.y16_bits(s), dw.device) for s in slots]
        slora.lora_apply_multi_y16(plan, slots, [t.data_ptr() for t in xs], [t.data_ptr() for t in y16])
        one = bits_to_device(w.y16_bits(5), dw.device)
        slora.lora_apply_multi_y16(plan, [5], [xs[5].data_ptr()], [one.data_ptr()])
        torch.cuda.synchronize()
        assert torch.equal(y16[5], one)
        with pytest.raises(slora.SloraError):  # nine slots are refused before anything is launched
            slora.lora_apply_multi(plan, slots + [0], [t.data_ptr() for t in xs + xs[:1]],
                                   [t.data_ptr() for t in ys + ys[:1]])
