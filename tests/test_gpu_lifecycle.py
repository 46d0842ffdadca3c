"""GPU tests of the per-batch life-cycle: a new plan every iteration (Sec. 4.1) must neither
allocate nor wait for the device once the library's recycled buffers exist, and everything a
plan enqueues must stay ordered when its buffers are reused or when streams change."""
import time

import numpy as np
import pytest
import torch

from paper_2311_03285_amd import slora, synth
from paper_2311_03285_amd.harness import DeviceWorkload, bits_to_device
from gpu_util import assert_close, oracle_slot
from test_gpu_parity import ragged_workload

pytestmark = pytest.mark.gpu


def batches(w, n, seed):
    """n re-drawn id vectors (pure decode) over the adapters of w, with their x bits."""
    g = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        ids = g.integers(-1, w.n_adapters, size=w.T).astype(np.int32)
        xb = synth.round_to_bits(g.standard_normal((w.T, w.H)).astype(np.float32), w.dtype)
        out.append((ids, xb))
    return out


def test_steady_state_cycle_allocates_nothing_and_stays_correct():
    w = ragged_workload(901, synth.F16, H=1000, n_pages=1500)
    with DeviceWorkload(w, real_adapters="all") as dw:
        st = torch.cuda.Stream()
        todo = batches(w, 12, 5)
        xs = [bits_to_device(xb, dw.device) for _, xb in todo]
        ys = [torch.zeros((w.T, w.H), dtype=torch.float32, device=dw.device) for _ in todo]
        torch.cuda.synchronize()
        stats = []
        for it in range(60):                    # five passes over the twelve batches
            k = it % len(todo)
            if it >= 48:
                with torch.cuda.stream(st):
                    ys[k].zero_()
            ids = todo[k][0]
            plan = slora.batch_plan(dw.pool, ids, None)
            slora.lora_apply(plan, 0, xs[k].data_ptr(), ys[k].data_ptr(), st)
            slora.plan_destroy(plan)
            if it % 3 == 2:
                st.synchronize()        # at most three batches in flight: finished sets are handed out again
            stats.append(slora.pool_stats(dw.pool))
        torch.cuda.synchronize()
        # every set in the rotation has its buffers after a while: no further set or allocation
        assert stats[-1]["allocations"] == stats[39]["allocations"], stats[::6]
        assert stats[-1]["sets_made"] == stats[39]["sets_made"], stats[::6]
        for k, (ids, xb) in enumerate(todo):
            ref = oracle_slot(w, 0, ids=ids, x_bits=xb, y_in=np.zeros((w.T, w.H), np.float32))
            assert_close(ys[k].cpu().numpy(), ref, f"batch {k}", rel_bar=5e-6)


def test_one_shot_calls_back_to_back_without_waiting():
    w = ragged_workload(902, synth.BF16, H=512, n_pages=1200)
    with DeviceWorkload(w, real_adapters="all") as dw:
        st = torch.cuda.Stream()
        todo = batches(w, 6, 9)
        xs = [bits_to_device(xb, dw.device) for _, xb in todo]
        ys = [torch.zeros((w.T, w.H), dtype=torch.float32, device=dw.device) for _ in todo]
        torch.cuda.synchronize()
        for k, (ids, _) in enumerate(todo):     # no synchronisation between the calls
            slora.lora_shrink_expand(dw.pool, 0, xs[k].data_ptr(), ids, None, ys[k].data_ptr(), st)
        torch.cuda.synchronize()
        for k, (ids, xb) in enumerate(todo):
            ref = oracle_slot(w, 0, ids=ids, x_bits=xb, y_in=np.zeros((w.T, w.H), np.float32))
            assert_close(ys[k].cpu().numpy(), ref, f"one-shot {k}", rel_bar=5e-6)


def test_plan_destroy_does_not_wait_for_another_stream():
    w = ragged_workload(903, synth.F16, H=512, n_pages=1200)
    with DeviceWorkload(w, real_adapters="all") as dw:
        a, b = torch.cuda.Stream(), torch.cuda.Stream()
        x = bits_to_device(w.x_bits(0), dw.device)
        y = torch.from_numpy(w.y_in(0)).to(dw.device)
        warm = slora.batch_plan(dw.pool, w.ids, None)
        slora.lora_apply(warm, 0, x.data_ptr(), y.data_ptr(), a)
        slora.plan_destroy(warm)
        torch.cuda.synchronize()
        y.copy_(torch.from_numpy(w.y_in(0)))
        torch.cuda.synchronize()
        # a kernel that spins for about 0.4 s on stream b (cycle count calibrated on this machine)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        with torch.cuda.stream(b):
            e0.record(b)
            torch.cuda._sleep(10_000_000)
            e1.record(b)
        b.synchronize()
        cycles = int(10_000_000 * 400.0 / max(e0.elapsed_time(e1), 1e-3))
        busy_done = torch.cuda.Event()
        with torch.cuda.stream(b):
            torch.cuda._sleep(cycles)
            busy_done.record(b)
        t0 = time.perf_counter()
        plan = slora.batch_plan(dw.pool, w.ids, None)
        slora.lora_apply(plan, 0, x.data_ptr(), y.data_ptr(), a)
        slora.plan_destroy(plan)
        dt = time.perf_counter() - t0
        still_running = not busy_done.query()
        a.synchronize()                          # stream a finishes while b still spins
        a_done_first = not busy_done.query()
        torch.cuda.synchronize()
        assert still_running, f"plan / apply / destroy took {dt * 1e3:.1f} ms and outlasted the other stream's kernel"
        assert a_done_first, "the apply waited for the other stream's kernel"
        assert_close(y.cpu().numpy(), oracle_slot(w, 0), "apply beside a busy stream", rel_bar=5e-6)


def test_one_plan_on_two_streams_is_ordered():
    """Applies of one plan share its v scratch; the library orders them when the stream changes."""
    w = ragged_workload(904, synth.F16, H=1000, n_pages=1500, n_slots=2)
    with DeviceWorkload(w, real_adapters="all") as dw:
        a, b = torch.cuda.Stream(), torch.cuda.Stream()
        plan = dw.plan(seg_offsets=None)
        xs = [bits_to_device(w.x_bits(s), dw.device) for s in (0, 1)]
        for rep in range(3):
            ys = [torch.from_numpy(w.y_in(s)).to(dw.device) for s in (0, 1)]
            torch.cuda.synchronize()
            slora.lora_apply(plan, 0, xs[0].data_ptr(), ys[0].data_ptr(), a)
            slora.lora_apply(plan, 1, xs[1].data_ptr(), ys[1].data_ptr(), b)
            torch.cuda.synchronize()
            for s in (0, 1):
                assert_close(ys[s].cpu().numpy(), oracle_slot(w, s), f"slot {s} rep {rep}", rel_bar=5e-6)


def test_write_pages_is_asynchronous_and_copies_its_host_arguments():
    H, n = 512, 300
    dev = torch.device("cuda:0")
    pool_t = torch.zeros((1024, H), dtype=torch.int16, device=dev)
    pool = slora.pool_init(H, 1024, synth.F16, pool_t.data_ptr(), 1, 8)
    g = np.random.default_rng(3)
    st = torch.cuda.Stream()
    idx = g.permutation(1024)[:n].astype(np.int32)
    src = g.integers(0, 0x7BFF, size=(n, H)).astype(np.uint16)
    keep_idx, keep_src = idx.copy(), src.copy()
    slora.pool_write_pages(pool, idx, src, False, st)
    idx[:] = 0                                    # the caller's arrays are free again at once
    src[:] = 0xFFFF
    st.synchronize()
    got = pool_t.cpu().numpy().view(np.uint16)
    assert np.array_equal(got[keep_idx], keep_src)
    untouched = np.ones(1024, dtype=bool)
    untouched[keep_idx] = False
    assert not got[untouched].any()
    # second write of other pages, device source, same stream: the first set is recycled
    before = slora.pool_stats(pool)
    d_src = torch.from_numpy(keep_src[:50].view(np.int16)).to(dev)
    idx2 = np.nonzero(untouched)[0][:50].astype(np.int32)
    slora.pool_write_pages(pool, idx2, d_src.data_ptr(), True, st)
    st.synchronize()
    assert np.array_equal(pool_t.cpu().numpy().view(np.uint16)[idx2], keep_src[:50])
    assert slora.pool_stats(pool)["sets_made"] == before["sets_made"]
    slora.pool_destroy(pool)
