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


# ------------------------------------------------------------------ H shared out over workgroups
def split(pool, nbytes=4096, min_h=128):
    """Force the MFMA shrink to cut every tile's H range into many small shares."""
    slora.set_option(pool, "mfma_split_bytes", nbytes)
    slora.set_option(pool, "mfma_split_min_h", min_h)


@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
@pytest.mark.parametrize("H", [320, 1000, 4096])
def test_shares_of_H_add_up_to_the_oracle(dtype, H):
    w = prefill_workload(500 + H, dtype, H=H)
    with DeviceWorkload(w, real_adapters="all", max_rank=160) as dw:
        route(dw.pool, MFMA_ALL)
        whole = gpu_slot(dw, 0, dw.plan())
        split(dw.pool)
        plan = dw.plan()
        info = slora.plan_info(plan)
        assert info["split_tiles"] > 0 and info["mfma_shrink_items"] >= 2 * info["split_tiles"]
        for slot in range(w.n_slots):
            got = gpu_slot(dw, slot, plan)
            rel, _ = assert_close(got, oracle_slot(w, slot), f"split H={H} slot={slot}")
            assert rel <= 5e-6, rel
        rel, _ = errors(gpu_slot(dw, 0, plan), whole.astype(np.float64))
        assert rel <= 2e-6                      # the two summation orders agree to rounding


@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
def test_shares_of_H_integer_inputs_bit_exact_and_deterministic(dtype):
    w = prefill_workload(520, dtype, H=1000, int_valued=True)
    with DeviceWorkload(w, real_adapters="all", max_rank=160) as dw:
        route(dw.pool, MFMA_ALL)
        split(dw.pool)
        plan = dw.plan()
        assert np.array_equal(gpu_slot(dw, 1, plan).astype(np.float64), oracle_slot(w, 1))
    w = prefill_workload(521, dtype, H=4096, n_slots=4, n_pages=4000)
    with DeviceWorkload(w, real_adapters="all", max_rank=160) as dw:
        route(dw.pool, MFMA_ALL)
        split(dw.pool, 16384, 128)
        plan = dw.plan()
        # whichever share arrives last adds the shares in the same order: the same bits every time,
        # in one launch for four slots as in four launches
        first = [gpu_slot(dw, s, plan) for s in range(4)]
        for rep in range(4):
            xs = [dw.x_dev(s) for s in range(4)]
            ys = [dw.y_dev(s) for s in range(4)]
            slora.lora_apply_multi(plan, [0, 1, 2, 3], [t.data_ptr() for t in xs], [t.data_ptr() for t in ys])
            torch.cuda.synchronize()
            for s in range(4):
                assert np.array_equal(ys[s].cpu().numpy(), first[s]), (rep, s)


@pytest.mark.parametrize("log2_scale", [-12, -6, 6, 12])
def test_fp16_v_far_from_unit_scale(log2_scale):
    """The 16-bit pieces that carry v into the MFMA expand must hold fp32 precision whatever the
    magnitude of v (activations far from N(0,1)): against the oracle on the delta alone, and
    against the vector kernels on the same batch."""
    w = prefill_workload(530, synth.F16, H=1000, y_zero=True)
    from paper_2311_03285_amd.synth import round_to_bits
    g = np.random.default_rng(530 + log2_scale)
    xb = round_to_bits(g.standard_normal((w.T, w.H)).astype(np.float32) * np.float32(2.0 ** log2_scale), w.dtype)
    ref = oracle_slot(w, 0, x_bits=xb)
    with DeviceWorkload(w, real_adapters="all", max_rank=160) as dw:
        outs = {}
        for name, thr in (("mfma", MFMA_ALL), ("vec", VEC_ONLY)):
            route(dw.pool, thr)
            outs[name] = gpu_slot(dw, 0, dw.plan(), x_bits=xb)
            assert np.isfinite(outs[name]).all()
            rel, _ = errors(outs[name], ref)
            assert rel <= 5e-6, (name, log2_scale, rel)
        split(dw.pool)
        route(dw.pool, MFMA_ALL)
        rel, _ = errors(gpu_slot(dw, 0, dw.plan(), x_bits=xb), ref)
        assert rel <= 5e-6, ("mfma, shared out", log2_scale, rel)


# ------------------------------------------------------------------ invariances on the MFMA path
@pytest.mark.parametrize("shares", [False, True])
def test_mfma_page_placement_invariance(shares):
    """Same weights at other page indices: no reduction order depends on page numbers, so the
    MFMA path too gives bit-identical results."""
    w1 = prefill_workload(540, synth.F16, H=512)
    w2 = prefill_workload(540, synth.F16, H=512, n_pages=3700)
    w2.page_idx = [(p.astype(np.int64) * 2 + 1).astype(np.int32) for p in w1.page_idx]
    outs = []
    for w in (w1, w2):
        with DeviceWorkload(w, real_adapters="all", max_rank=160) as dw:
            route(dw.pool, MFMA_ALL)
            if shares:
                split(dw.pool)
            outs.append(gpu_slot(dw, 1))
    assert np.array_equal(outs[0], outs[1])


@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
def test_mfma_request_permutation(dtype):
    """Requests in another order (tokens of a request stay together): every output row is the
    same up to the rounding of a different tile alignment, and right against the oracle."""
    w = prefill_workload(550, dtype, H=512)
    n_seg = w.seg_offsets.size - 1
    order = np.random.default_rng(2).permutation(n_seg)
    rows = np.concatenate([np.arange(w.seg_offsets[s], w.seg_offsets[s + 1]) for s in order])
    seg2 = np.concatenate([[0], np.cumsum(np.diff(w.seg_offsets)[order])]).astype(np.int32)
    with DeviceWorkload(w, real_adapters="all", max_rank=160) as dw:
        route(dw.pool, MFMA_ALL)
        a = gpu_slot(dw, 0)
        p2 = dw.plan(ids=w.ids[rows], seg_offsets=seg2)
        b = gpu_slot(dw, 0, p2, x_bits=w.x_bits(0)[rows], y_in=w.y_in(0)[rows])
        assert_close(b, oracle_slot(w, 0)[rows], "permuted requests")
        rel, _ = errors(b, a[rows].astype(np.float64))
        assert rel <= 1e-6
        # token order scrambled inside the batch as well (a pure-decode description of the same ids)
        perm = np.random.default_rng(3).permutation(w.T)
        p3 = dw.plan(ids=w.ids[perm], seg_offsets=None)
        c = gpu_slot(dw, 0, p3, x_bits=w.x_bits(0)[perm], y_in=w.y_in(0)[perm])
        assert_close(c, oracle_slot(w, 0)[perm], "permuted tokens")
        rel, _ = errors(c, a[perm].astype(np.float64))
        assert rel <= 1e-6


# ------------------------------------------------------------------ every slot of the timed shapes
def _all_slots(n):
    """Every slot of a full-size configuration, eight slots per launch pair as the bench times
    it, against the oracle on a seeded sample of tokens (the oracle computes them one by one)."""
    w = synth.config(n)
    slots = list(range(w.n_slots))
    act = np.nonzero(w.ids >= 0)[0]
    samp = np.sort(np.random.default_rng(n).choice(act, size=min(act.size, 96), replace=False))
    ids_s = np.full_like(w.ids, -1)
    ids_s[samp] = w.ids[samp]
    with DeviceWorkload(w, real_adapters=np.unique(w.ids[samp]), slots=slots) as dw:
        plan = dw.plan()
        for g0 in range(0, len(slots), slora.MAX_MULTI):
            grp = slots[g0:g0 + slora.MAX_MULTI]
            xs = [dw.x_dev(s) for s in grp]
            ys = [dw.y_dev(s) for s in grp]
            slora.lora_apply_multi(plan, grp, [t.data_ptr() for t in xs], [t.data_ptr() for t in ys])
            torch.cuda.synchronize()
            for s, t in zip(grp, ys):
                got = t.cpu().numpy()[samp]
                assert np.isfinite(got).all(), s
                ref = oracle_slot(w, s, ids=ids_s)[samp]
                rel, _ = assert_close(got, ref, f"cfg{n} slot {s}")
                assert rel <= 5e-6, (s, rel)


def test_config3_every_slot():
    _all_slots(3)


def test_config5_every_slot():
    _all_slots(5)


# ------------------------------------------------------------------ HIP graph capture of every kernel
@pytest.mark.parametrize("entry", ["multi", "static"])
@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
def test_mixed_batch_captured_in_a_hip_graph(dtype, entry):
    """A mixed batch whose apply launches every kernel the library has - the MFMA shrink with
    shared-out tiles, the join of their partial sums, the one-launch decode kernel, the
    two-stage vector kernels (a nine-token group), the MFMA expand - captured in a HIP graph
    through the allocating entry point (scratch sized by an eager call first) and through the
    one that allocates nothing.  Every replay, with the program's own eager work in between,
    must reproduce the eager result bit for bit; the eager result meets the oracle."""
    lens = (1, 1, 2, 4, 9, 1, 3, 40, 130, 1, 1, 100)
    ranks = (8, 16, 64, 128, 33, 160, 7, 32, 1, 5, 17, 96)
    seg = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    seg_ad = np.random.default_rng(2600 + dtype).permutation(len(ranks))
    seg_ad[5] = -1                                       # one decode token without adapter
    ids = np.repeat(seg_ad, lens).astype(np.int32)
    w = synth.make_workload("graph-mixed", 2600 + dtype, 1024, dtype, 3000, 2, ranks, ids, seg)
    with DeviceWorkload(w, real_adapters="all", max_rank=160) as dw:
        route(dw.pool, 16)
        slora.set_option(dw.pool, "mfma_split_bytes", 1 << 16)
        slora.set_option(dw.pool, "mfma_split_min_h", 128)
        slora.set_option(dw.pool, "fuse_decode", 2)
        plan = dw.plan()
        info = slora.plan_info(plan)
        assert info["split_tiles"] > 0 and info["groups_fused"] > 0 and info["groups_mfma"] > 0
        assert info["groups_fused"] < info["groups_vec"]          # the nine-token group stays on two kernels
        apply = slora.lora_apply_multi if entry == "multi" else slora.lora_apply_multi_static
        x = [dw.x_dev(0), dw.x_dev(1)]
        y0 = [dw.y_dev(0), dw.y_dev(1)]
        y = [t.clone() for t in y0]
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            apply(plan, [0, 1], [t.data_ptr() for t in x], [t.data_ptr() for t in y], torch.cuda.current_stream())
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        eager = [t.cpu().numpy() for t in y]
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            apply(plan, [0, 1], [t.data_ptr() for t in x], [t.data_ptr() for t in y], torch.cuda.current_stream())
        for rep in range(4):
            for k in range(2):
                y[k].copy_(y0[k])               # eager work between the replays
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            for k in range(2):
                assert np.array_equal(y[k].cpu().numpy(), eager[k]), (rep, k)
        for k in range(2):
            assert_close(eager[k], oracle_slot(w, k), f"graph slot {k}", rel_bar=5e-6)
