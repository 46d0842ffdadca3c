"""GPU parity: the HIP path, called through the C ABI, against the CPU fp64 oracle.

Tolerance (written here as the benchmark spec states it): relative L2 error <= 1e-3 and max-abs
error <= 1e-2 on N(0,1) activations, checked on the outputs and again on the delta alone
(y_in = 0) so that the error is not hidden behind y.  Page gathers and integer-valued inputs
must match bit for bit.
"""
import numpy as np
import pytest
import torch

from paper_2311_03285_amd import slora, synth
from paper_2311_03285_amd.harness import DeviceWorkload, bits_to_device
from gpu_util import (MAX_ABS_BAR, REL_L2_BAR, REL_L2_EXPECTED, assert_close, errors, gpu_slot, oracle_slot)

pytestmark = pytest.mark.gpu

VEC_ONLY = 1 << 40


def ragged_workload(seed, dtype, H=1000, T=37, ranks=(1, 3, 0, 5, 17, 8, 64, 33), n_slots=2, n_pages=700, **kw):
    g = np.random.default_rng(seed)
    ids = g.integers(0, len(ranks), size=T)
    ids[g.integers(0, T, size=3)] = -1
    ids[5:14] = 4                                   # a 9-token group: several token chunks
    return synth.make_workload("ragged", seed, H, dtype, n_pages, n_slots, ranks, ids, **kw)


# ------------------------------------------------------------------ gather (bit-exact)
@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
def test_gather_bit_exact(dtype):
    w = ragged_workload(101, dtype)
    with DeviceWorkload(w, real_adapters="all") as dw:
        for a in range(w.n_adapters):
            for s in range(w.n_slots):
                for which in (0, 1):
                    got = dw.gather(a, s, which)
                    assert np.array_equal(got, w.weight_bits(a, s, which)), (a, s, which)
        # pages nobody owns still hold the canary: the scatter wrote only where it was told to
        pool = dw.pool_t.cpu().numpy().view(np.uint16)
        free = np.ones(w.n_pages, bool)
        free[w.owned_pages()] = False
        assert np.all(pool[free] == synth.nan_bits(dtype))


# ------------------------------------------------------------------ configs 1 and 2 (decode)
@pytest.mark.parametrize("n", [1, 2])
@pytest.mark.parametrize("y_zero", [False, True])
def test_decode_configs(n, y_zero):
    w = synth.config(n, y_zero=y_zero)
    with DeviceWorkload(w, real_adapters="all" if n == 1 else "used") as dw:
        got = gpu_slot(dw, 0)
        ref = oracle_slot(w, 0)
        rel, mx = assert_close(got, ref, f"cfg{n} y_zero={y_zero}")
        assert rel <= REL_L2_EXPECTED, rel


def test_one_shot_call_matches_plan_apply():
    w = synth.config(1)
    with DeviceWorkload(w, real_adapters="all") as dw:
        a = gpu_slot(dw, 0)
        x, y = dw.x_dev(0), dw.y_dev(0)
        slora.lora_shrink_expand(dw.pool, 0, x.data_ptr(), w.ids, None, y.data_ptr())
        assert np.array_equal(a, y.cpu().numpy())


# ------------------------------------------------------------------ ragged shapes, both dtypes
@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
@pytest.mark.parametrize("H", [64, 1000, 5120])
def test_ragged_vector_path(dtype, H):
    w = ragged_workload(200 + H, dtype, H=H, n_pages=900)
    with DeviceWorkload(w, real_adapters="all") as dw:
        slora.set_option(dw.pool, "mfma_min_tokens", VEC_ONLY)
        for slot in range(w.n_slots):
            got = gpu_slot(dw, slot)
            ref = oracle_slot(w, slot)
            rel, mx = assert_close(got, ref, f"H={H} slot={slot}")
            assert rel <= REL_L2_EXPECTED, rel
            yi = w.y_in(slot)
            untouched = (w.ids < 0) | (w.ranks[np.maximum(w.ids, 0)] == 0)
            assert np.array_equal(got[untouched], yi[untouched])      # bit-for-bit


# ------------------------------------------------------------------ exact cases
@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
def test_integer_inputs_are_bit_exact(dtype):
    """Small-integer x, A, B, y: every partial sum is an integer below 2^24, so any order of
    fp32 accumulation is exact and the GPU must equal the fp64 oracle bit for bit."""
    w = ragged_workload(301, dtype, H=512, int_valued=True)
    with DeviceWorkload(w, real_adapters="all") as dw:
        slora.set_option(dw.pool, "mfma_min_tokens", VEC_ONLY)
        for slot in range(w.n_slots):
            got = gpu_slot(dw, slot)
            ref = oracle_slot(w, slot)
            assert np.array_equal(got.astype(np.float64), ref)


def test_zero_B_pages_leave_y_bitwise_unchanged():
    w = ragged_workload(302, synth.F16, H=512)
    with DeviceWorkload(w, real_adapters="all") as dw:
        slora.set_option(dw.pool, "mfma_min_tokens", VEC_ONLY)
        pages = np.concatenate([w.page_idx[a][0, 1] for a in range(w.n_adapters)])
        slora.pool_write_pages(dw.pool, pages, np.zeros((pages.size, w.H), np.uint16), False)
        yi = w.y_in(0)
        yi[yi == 0] = 0.0           # no negative zeros: -0 + 0 = +0 would differ in the sign bit
        got = gpu_slot(dw, 0, y_in=yi)
        assert np.array_equal(got.view(np.uint32), yi.view(np.uint32))


# ------------------------------------------------------------------ invariants on the GPU
def test_run_to_run_determinism_and_multi_slot():
    w = ragged_workload(303, synth.BF16, H=1000)
    with DeviceWorkload(w, real_adapters="all") as dw:
        slora.set_option(dw.pool, "mfma_min_tokens", VEC_ONLY)
        plan = dw.plan()
        a0, a1 = gpu_slot(dw, 0, plan), gpu_slot(dw, 1, plan)
        assert np.array_equal(a0, gpu_slot(dw, 0, plan))
        xs = [dw.x_dev(0), dw.x_dev(1)]
        ys = [dw.y_dev(0), dw.y_dev(1)]
        slora.lora_apply_multi(plan, [0, 1], [t.data_ptr() for t in xs], [t.data_ptr() for t in ys])
        torch.cuda.synchronize()
        assert np.array_equal(ys[0].cpu().numpy(), a0) and np.array_equal(ys[1].cpu().numpy(), a1)
        # the two stages on their own give the same bits
        ys2 = [dw.y_dev(0), dw.y_dev(1)]
        slora.lora_shrink(plan, [0, 1], [t.data_ptr() for t in xs])
        slora.lora_expand(plan, [0, 1], [t.data_ptr() for t in ys2])
        torch.cuda.synchronize()
        assert np.array_equal(ys2[0].cpu().numpy(), a0) and np.array_equal(ys2[1].cpu().numpy(), a1)


def test_page_placement_invariance_on_gpu():
    """Same weights at other page indices: the reduction order does not depend on page
    numbers, so the result is bit-identical."""
    w1 = ragged_workload(304, synth.F16, H=512)
    w2 = ragged_workload(304, synth.F16, H=512, n_pages=1400)
    w2.page_idx = [(p.astype(np.int64) * 2 + 1).astype(np.int32) for p in w1.page_idx]
    outs = []
    for w in (w1, w2):
        with DeviceWorkload(w, real_adapters="all") as dw:
            slora.set_option(dw.pool, "mfma_min_tokens", VEC_ONLY)
            outs.append(gpu_slot(dw, 0))
    assert np.array_equal(outs[0], outs[1])


def test_batch_permutation_on_gpu():
    w = ragged_workload(305, synth.F16, H=512)
    perm = np.random.default_rng(1).permutation(w.T)
    with DeviceWorkload(w, real_adapters="all") as dw:
        slora.set_option(dw.pool, "mfma_min_tokens", VEC_ONLY)
        a = gpu_slot(dw, 0)
        p2 = dw.plan(ids=w.ids[perm], seg_offsets=None)
        b = gpu_slot(dw, 0, p2, x_bits=w.x_bits(0)[perm], y_in=w.y_in(0)[perm])
        ref = oracle_slot(w, 0)
        assert_close(b, ref[perm], "permuted")
        rel, _ = errors(b, a[perm].astype(np.float64))
        assert rel <= 1e-6


def test_empty_batch_and_all_tokens_without_adapter():
    w = ragged_workload(306, synth.F16, H=512)
    with DeviceWorkload(w, real_adapters="all") as dw:
        p0 = dw.plan(ids=np.zeros(0, np.int32), seg_offsets=None)
        slora.lora_apply(p0, 0, dw.x_dev(0).data_ptr(), dw.y_dev(0).data_ptr())
        ids = np.full(w.T, -1, np.int32)
        p1 = dw.plan(ids=ids, seg_offsets=None)
        got = gpu_slot(dw, 0, p1)
        assert np.array_equal(got, w.y_in(0))


# ------------------------------------------------------------------ extreme shapes
@pytest.mark.parametrize("path", ["vec", "mfma"])
def test_largest_page_size(path):
    """H = 32768 (the largest page the pool accepts): one x row fills the 64 KiB the vector
    shrink may stage, so multi-token groups are cut into single-token items."""
    g = np.random.default_rng(7)
    ranks = (8, 40)
    ids = np.array([0, 1, 1, 0, 1, -1, 1, 1], dtype=np.int32)
    w = synth.make_workload("max-H", 901, 32768, synth.F16, 128, 1, ranks, ids)
    with DeviceWorkload(w, real_adapters="all") as dw:
        slora.set_option(dw.pool, "mfma_min_tokens", VEC_ONLY if path == "vec" else 1)
        slora.set_option(dw.pool, "mfma_min_tiles", 1)
        got = gpu_slot(dw, 0)
        rel, mx = assert_close(got, oracle_slot(w, 0), f"H=32768 {path}")
        assert rel <= 5e-6


@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
@pytest.mark.parametrize("path", ["vec", "mfma"])
def test_largest_rank(dtype, path):
    """rank 1024 (the largest max_rank): 16 windows of 64 ranks in the vector expand, 16 rank
    chunks in the MFMA shrink, 32 stages in the MFMA expand."""
    lens = [3, 40]
    ids = np.repeat([0, 1], lens).astype(np.int32)
    seg = np.array([0, 3, 43], dtype=np.int32)
    w = synth.make_workload("max-rank", 902, 256, dtype, 4200, 1, (1024, 1000), ids, seg)
    with DeviceWorkload(w, real_adapters="all", max_rank=1024) as dw:
        slora.set_option(dw.pool, "mfma_min_tokens", VEC_ONLY if path == "vec" else 1)
        slora.set_option(dw.pool, "mfma_min_tiles", 1)
        got = gpu_slot(dw, 0)
        rel, mx = assert_close(got, oracle_slot(w, 0), f"rank 1024 {path}")
        assert rel <= 5e-6


# ------------------------------------------------------------------ adapters come and go
def test_unload_and_reload_reuses_pages_and_table_slots():
    """Adapters are swapped between batches (the paper fetches the adapters of each batch into
    the pool): after an unload the freed pages and the freed run of the page-list table are
    taken by other adapters, old plans are refused, new plans see the new lists."""
    import dataclasses
    w = ragged_workload(307, synth.F16, H=512, ranks=(4, 16, 8, 16, 12), n_slots=1, n_pages=200)
    with DeviceWorkload(w, real_adapters="all", mark_kv=False, max_rank=32) as dw:
        old_plan = dw.plan()
        before = gpu_slot(dw, 0, old_plan)
        assert_close(before, oracle_slot(w, 0), "before the swap")
        # adapter 1 (rank 16) leaves; adapter 3's twin 7 (rank 16: same table run length) and a
        # rank-24 adapter 1 arrive on the freed pages plus fresh ones
        freed = w.page_idx[1].reshape(-1)
        slora.adapter_unload(dw.pool, 1)
        with pytest.raises(slora.SloraError) as e:
            slora.lora_apply(old_plan, 0, dw.x_dev(0).data_ptr(), dw.y_dev(0).data_ptr())
        assert e.value.code == slora.EBUSY
        used = set(int(p) for p in w.owned_pages())
        fresh = [p for p in range(w.n_pages) if p not in used][:48 + 32 - freed.size]
        pages = np.concatenate([freed, np.array(fresh, np.int32)]).astype(np.int32)
        ranks2 = np.concatenate([w.ranks, [0, 0, 16]]).astype(np.int32)         # ids 5, 6 unused
        ranks2[1] = 24
        page_idx2 = list(w.page_idx) + [np.zeros((1, 2, 0), np.int32)] * 2 + [pages[48:80].reshape(1, 2, 16)]
        page_idx2[1] = pages[:48].reshape(1, 2, 24)
        ids2 = w.ids.copy()
        ids2[ids2 == 3] = 7
        w2 = dataclasses.replace(w, ranks=ranks2, page_idx=page_idx2, ids=ids2)
        for a in (1, 7):
            slora.adapter_load(dw.pool, a, int(ranks2[a]), w2.adapter_page_list(a))
            for which in (0, 1):
                slora.pool_write_pages(dw.pool, w2.page_idx[a][0, which], w2.weight_bits(a, 0, which), False)
        dw.w = w2
        got = gpu_slot(dw, 0, dw.plan(ids=ids2, seg_offsets=None))
        assert_close(got, oracle_slot(w2, 0), "after the swap")
        assert np.array_equal(dw.gather(7, 0, 1), w2.weight_bits(7, 0, 1))


# ------------------------------------------------------------------ HIP graph capture
def test_apply_can_be_captured_in_a_hip_graph():
    """A serving loop replays the decode step as a HIP graph: once the plan's scratch exists, an
    apply makes no allocation, copy or synchronisation, only kernel launches on the caller's
    stream.  Every replay must reproduce the eager result bit for bit (y is reset in between by
    eager work of the program itself)."""
    w = ragged_workload(308, synth.F16, H=1024, T=48)
    with DeviceWorkload(w, real_adapters="all") as dw:
        plan = dw.plan()
        x = [dw.x_dev(0), dw.x_dev(1)]
        y0 = [dw.y_dev(0), dw.y_dev(1)]
        y = [t.clone() for t in y0]
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):           # eager warm-up on the capture stream: sizes the scratch
            slora.lora_apply_multi(plan, [0, 1], [t.data_ptr() for t in x], [t.data_ptr() for t in y],
                                   torch.cuda.current_stream())
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        eager = [t.cpu().numpy() for t in y]
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            slora.lora_apply_multi(plan, [0, 1], [t.data_ptr() for t in x], [t.data_ptr() for t in y],
                                   torch.cuda.current_stream())
        for rep in range(4):
            for k in range(2):
                y[k].copy_(y0[k])               # eager work between the replays
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            for k in range(2):
                assert np.array_equal(y[k].cpu().numpy(), eager[k]), (rep, k)
        assert_close(eager[0], oracle_slot(w, 0), "graph slot 0")


def test_graph_replay_survives_table_growth():
    """After the capture, more adapters are loaded (the device page-list table outgrows its
    allocation) and the plan is applied with more slots than before (so does the v scratch): the
    tables the captured launches point at must still be there, and still right, on replay."""
    w = ragged_workload(309, synth.BF16, H=512, T=40, n_pages=8000)
    with DeviceWorkload(w, real_adapters="all", mark_kv=False, max_rank=64) as dw:
        plan = dw.plan()
        x, y0 = dw.x_dev(0), dw.y_dev(0)
        y = y0.clone()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            slora.lora_apply(plan, 0, x.data_ptr(), y.data_ptr(), torch.cuda.current_stream())
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        eager = y.cpu().numpy()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            slora.lora_apply(plan, 0, x.data_ptr(), y.data_ptr(), torch.cuda.current_stream())
        for a in range(100, 124):                       # 24 x 256 list entries: past the first 4096
            slora.adapter_alloc(dw.pool, a, 64, w.n_slots)
        xs, ys = [dw.x_dev(0), dw.x_dev(1)], [dw.y_dev(0), dw.y_dev(1)]
        slora.lora_apply_multi(plan, [0, 1], [t.data_ptr() for t in xs], [t.data_ptr() for t in ys])
        torch.cuda.synchronize()
        assert np.array_equal(ys[0].cpu().numpy(), eager)      # the regrown tables give the same bits
        for rep in range(3):
            y.copy_(y0)
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            assert np.array_equal(y.cpu().numpy(), eager), rep
        assert_close(eager, oracle_slot(w, 0), "graph after growth")


def test_projections_sharing_one_x_buffer():
    """q, k, v of a layer read the same activations: one call over three slots with the same x
    pointer gives, per slot, the bits of that slot applied on its own (vector and MFMA paths)."""
    w = ragged_workload(311, synth.F16, H=1024, n_slots=3, n_pages=1000)
    for min_tok in (VEC_ONLY, 1):
        with DeviceWorkload(w, real_adapters="all") as dw:
            slora.set_option(dw.pool, "mfma_min_tokens", min_tok)
            slora.set_option(dw.pool, "mfma_min_tiles", 1)
            plan = dw.plan()
            x = dw.x_dev(0)
            single = []
            for s in range(3):
                y = dw.y_dev(s)
                slora.lora_apply(plan, s, x.data_ptr(), y.data_ptr())
                single.append(y)
            ys = [dw.y_dev(s) for s in range(3)]
            slora.lora_apply_multi(plan, [0, 1, 2], [x.data_ptr()] * 3, [t.data_ptr() for t in ys])
            torch.cuda.synchronize()
            for s in range(3):
                assert np.array_equal(ys[s].cpu().numpy(), single[s].cpu().numpy())
                # and against the oracle: slot s's weights, slot 0's activations
                assert_close(ys[s].cpu().numpy(), oracle_slot(w, s, x_bits=w.x_bits(0)), f"shared x, slot {s}")


# ------------------------------------------------------------------ seeded random shapes
@pytest.mark.parametrize("seed", range(12))
def test_random_shapes_against_the_oracle(seed):
    """Seeded random batches inside the documented limits: H any multiple of 8 from 64 up, ranks
    from 0 to 96 (two rank windows of the vector expand, two rank chunks of the MFMA shrink),
    segments of 1 to 150 tokens, tokens without adapter, either storage type, the scheduler left
    to route by itself or forced to one kernel family; fp32 and 16-bit y."""
    g = np.random.default_rng(9000 + seed)
    H = int(g.choice([64, 72, 200, 512, 1000, 1536, 2048, 4104]))
    dtype = int(g.integers(0, 2))
    n_ad = int(g.integers(1, 9))
    ranks = tuple(int(r) for r in g.choice([0, 1, 2, 7, 8, 16, 31, 33, 64, 65, 96], size=n_ad))
    n_seg = int(g.integers(1, 12))
    lens = [int(v) for v in g.choice([1, 1, 1, 2, 3, 5, 17, 32, 33, 64, 70, 150], size=n_seg)]
    seg = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    seg_ad = g.integers(-1, n_ad, size=n_seg)
    ids = np.repeat(seg_ad, lens).astype(np.int32)
    n_slots = 2
    n_pages = int(2 * n_slots * 2 * sum(ranks) + 16)
    w = synth.make_workload("random", 9000 + seed, H, dtype, n_pages, n_slots, ranks, ids, seg)
    route_kind = ["auto", "vec", "mfma"][seed % 3]
    with DeviceWorkload(w, real_adapters="all", max_rank=96) as dw:
        if route_kind == "vec":
            slora.set_option(dw.pool, "mfma_min_tokens", VEC_ONLY)
        elif route_kind == "mfma":
            slora.set_option(dw.pool, "mfma_min_tokens", 1)
            slora.set_option(dw.pool, "mfma_min_tiles", 1)
        plan = dw.plan()
        untouched = (w.ids < 0) | (w.ranks[np.maximum(w.ids, 0)] == 0)
        for slot in range(n_slots):
            got = gpu_slot(dw, slot, plan)
            assert np.array_equal(got[untouched], w.y_in(slot)[untouched])
            if (~untouched).any():
                assert_close(got, oracle_slot(w, slot), f"seed {seed} H={H} ranks={ranks} lens={lens} {route_kind}")
        # the same batch with 16-bit y: within one 16-bit step of the fp32-y result, rounded
        yb = bits_to_device(w.y16_bits(0), dw.device)
        x = dw.x_dev(0)
        slora.lora_apply_multi_y16(plan, [0], [x.data_ptr()], [yb.data_ptr()])
        torch.cuda.synchronize()
        got16 = yb.cpu().numpy().view(np.uint16).reshape(w.T, H)
        assert np.array_equal(got16[untouched], w.y16_bits(0)[untouched])
        dec = (lambda b: b.view(np.float16).astype(np.float64)) if dtype == synth.F16 else \
              (lambda b: (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64))
        ref = oracle_slot(w, 0, y_in=dec(w.y16_bits(0)).astype(np.float32))
        tol = (2.0 ** -10 if dtype == synth.F16 else 2.0 ** -7) * np.maximum(np.abs(ref), 2.0 ** -14) + 1e-5
        assert np.all(np.abs(dec(got16) - ref) <= tol)


@pytest.mark.parametrize("seed", range(16))
def test_random_options_and_entry_points_against_the_oracle(seed):
    """Seeded random batches as above, with the tuning options drawn at random too (routing
    thresholds, share size and shortest share of the MFMA shrink, the one-launch decode rule,
    pages per vector-shrink item, tile grouping), one to four slots in one call in a random
    order, through a randomly chosen entry point: the multi-slot apply, the apply that
    allocates nothing, shrink and expand as two calls, or the one-shot call per slot.  None of
    this may change the result beyond rounding: every slot against the oracle at the regression
    bar, rows without an adapter bit for bit."""
    g = np.random.default_rng(77000 + seed)
    H = int(g.choice([64, 72, 200, 512, 1000, 1536, 2048, 4104]))
    dtype = int(g.integers(0, 2))
    n_ad = int(g.integers(1, 10))
    ranks = tuple(int(r) for r in g.choice([0, 1, 2, 7, 8, 16, 31, 32, 33, 64, 65, 96, 128, 129, 160], size=n_ad))
    n_seg = int(g.integers(1, 24))
    lens = [int(v) for v in g.choice([1, 1, 1, 1, 2, 3, 4, 5, 17, 32, 33, 64, 70, 127, 128, 129, 150], size=n_seg)]
    seg = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    ids = np.repeat(g.integers(-1, n_ad, size=n_seg), lens).astype(np.int32)
    n_slots = int(g.integers(1, 5))
    decode = bool(g.integers(0, 4) == 0)
    w = synth.make_workload("random-options", 77000 + seed, H, dtype, int(n_slots * 4 * sum(ranks) + 64), n_slots, ranks, ids,
                            None if decode else seg)
    opts = {"mfma_min_tokens": int(g.choice([1, 4, 16, VEC_ONLY])), "mfma_min_tiles": int(g.choice([1, 1, 4, 32])),
            "mfma_split_bytes": int(g.choice([1 << 16, 1 << 18, 1 << 20, 1 << 30])),
            "mfma_split_min_h": int(g.choice([128, 256, 1024])), "fuse_decode": int(g.integers(0, 3)),
            "shrink_pages": int(g.integers(1, 9)), "xcd_group": int(g.integers(0, 4))}
    entry = ["multi", "static", "two_calls", "one_shot"][int(g.integers(0, 4))]
    what = f"seed {seed} H={H} ranks={ranks} lens={lens} decode={decode} {opts} {entry}"
    with DeviceWorkload(w, real_adapters="all", max_rank=160) as dw:
        for k, v in opts.items():
            slora.set_option(dw.pool, k, v)
        st = torch.cuda.Stream()
        plan = dw.plan()
        slots = [int(s) for s in g.permutation(n_slots)]
        xs = [dw.x_dev(s) for s in slots]
        ys = [dw.y_dev(s) for s in slots]
        xp, yp = [x.data_ptr() for x in xs], [y.data_ptr() for y in ys]
        if entry == "multi":
            slora.lora_apply_multi(plan, slots, xp, yp, st)
        elif entry == "static":
            slora.lora_apply_multi_static(plan, slots, xp, yp, st)
        elif entry == "two_calls":
            slora.lora_shrink(plan, slots, xp, st)
            slora.lora_expand(plan, slots, yp, st)
        else:
            for s, x, y in zip(slots, xp, yp):
                slora.lora_shrink_expand(dw.pool, s, x, w.ids, w.seg_offsets, y, st)
        torch.cuda.synchronize()
        untouched = (w.ids < 0) | (w.ranks[np.maximum(w.ids, 0)] == 0)
        for s, y in zip(slots, ys):
            got = y.cpu().numpy()
            assert np.array_equal(got[untouched], w.y_in(s)[untouched]), what
            if (~untouched).any():
                assert_close(got, oracle_slot(w, s), f"slot {s} {what}", rel_bar=5e-6)


# ------------------------------------------------------------------ decode groups in one launch
@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
@pytest.mark.parametrize("H", [64, 1000, 5120, 6656, 8192])
def test_one_launch_decode_kernel_beside_the_two_kernels(dtype, H):
    """Adapter groups of at most four tokens through the kernel that does both stages in one
    launch (forced) against the two-kernel path on the same inputs (equal up to the order in
    which the small-batch expand adds its rank blocks), fp32 y and 16-bit y, several slots per
    launch, the entry point without allocation; and against the oracle."""
    w = ragged_workload(1300 + H, dtype, H=H, n_slots=3, n_pages=900)
    with DeviceWorkload(w, real_adapters="all") as dw:
        slora.set_option(dw.pool, "mfma_min_tokens", VEC_ONLY)
        outs = {}
        for mode in (0, 2):
            slora.set_option(dw.pool, "fuse_decode", mode)
            plan = dw.plan(seg_offsets=None)
            info = slora.plan_info(plan)
            assert (info["groups_fused"] > 0) == (mode == 2)
            assert info["groups_fused"] < info["groups"]          # the nine-token group stays on two kernels
            xs = [dw.x_dev(s) for s in range(3)]
            ys = [dw.y_dev(s) for s in range(3)]
            y16 = [bits_to_device(w.y16_bits(s), dw.device) for s in range(3)]
            slora.lora_apply_multi(plan, [0, 1, 2], [t.data_ptr() for t in xs], [t.data_ptr() for t in ys])
            slora.lora_apply_multi_y16(plan, [2, 0], [xs[2].data_ptr(), xs[0].data_ptr()],
                                       [y16[2].data_ptr(), y16[0].data_ptr()])
            st = dw.y_dev(1)
            slora.lora_apply_multi_static(plan, [1], [xs[1].data_ptr()], [st.data_ptr()])
            torch.cuda.synchronize()
            outs[mode] = ([t.cpu().numpy() for t in ys], [t.cpu().numpy() for t in y16], st.cpu().numpy())
            if mode == 2:       # v of the fused groups never reached memory: an expand alone is refused
                with pytest.raises(slora.SloraError) as e:
                    slora.lora_expand(plan, [1], [st.data_ptr()])
                assert e.value.code == slora.EINVAL
                slora.lora_shrink(plan, [1], [xs[1].data_ptr()])
                st2 = dw.y_dev(1)
                slora.lora_expand(plan, [1], [st2.data_ptr()])
                torch.cuda.synchronize()
                assert np.array_equal(st2.cpu().numpy(), outs[0][2])      # the two stages: the two-kernel bits
        for s in range(3):
            rel, _ = errors(outs[2][0][s], outs[0][0][s].astype(np.float64))
            assert rel <= 1e-6, (s, rel)
            differ = np.mean(outs[0][1][s] != outs[2][1][s])              # 16-bit y: the same rounding nearly everywhere
            assert differ <= 1e-3, (s, differ)
            rel, _ = assert_close(outs[2][0][s], oracle_slot(w, s), f"one-launch decode, slot {s}")
            assert rel <= REL_L2_EXPECTED
        assert np.array_equal(outs[2][2], outs[2][0][1])                  # static scratch entry: the same kernel


@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
def test_one_launch_decode_kernel_integer_inputs_bit_exact(dtype):
    w = ragged_workload(1400, dtype, H=5120, n_pages=900, int_valued=True)
    with DeviceWorkload(w, real_adapters="all") as dw:
        slora.set_option(dw.pool, "mfma_min_tokens", VEC_ONLY)
        slora.set_option(dw.pool, "fuse_decode", 2)
        plan = dw.plan(seg_offsets=None)
        assert slora.plan_info(plan)["groups_fused"] > 0
        for slot in range(w.n_slots):
            assert np.array_equal(gpu_slot(dw, slot, plan).astype(np.float64), oracle_slot(w, slot))
