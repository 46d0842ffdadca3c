"""GPU tests of the page allocator and the asynchronous adapter fetch: pages chosen by the
library (with KV pages scattered between them), weights copied from pinned host memory by a
kernel on a side stream while another batch computes, results against the oracle (which does
not depend on page placement) and gathered pages bit for bit."""
import numpy as np
import pytest
import torch

from paper_2311_03285_amd import slora, synth
from paper_2311_03285_amd.harness import bits_to_device
from gpu_util import assert_close, oracle_slot
from test_gpu_parity import ragged_workload

pytestmark = pytest.mark.gpu


def pinned_weights(w, a):
    """[n_slots, 2, r, H] 16-bit patterns of adapter a in pinned host memory."""
    r = int(w.ranks[a])
    t = torch.empty((w.n_slots, 2, max(r, 1), w.H), dtype=torch.int16).pin_memory()
    if r:
        for s in range(w.n_slots):
            for which in (0, 1):
                t[s, which] = torch.from_numpy(w.weight_bits(a, s, which).view(np.int16))
    return t


class FetchedPool:
    """A NaN-filled pool whose adapters are placed by the library's allocator."""

    def __init__(self, w, kv_every=3):
        self.w = w
        self.dev = torch.device("cuda:0")
        self.pool_t = torch.empty((w.n_pages, w.H), dtype=torch.int16, device=self.dev)
        nanv = synth.nan_bits(w.dtype)
        self.pool_t.fill_(nanv - 65536 if nanv >= 32768 else nanv)
        self.pool = slora.pool_init(w.H, w.n_pages, w.dtype, self.pool_t.data_ptr(), w.n_slots, int(w.ranks.max()))
        self.kv = np.arange(0, w.n_pages, kv_every, dtype=np.int32)          # KV pages interleaved
        slora.pool_mark_kv(self.pool, self.kv)
        self.host = {}
        self.pages = {}
        torch.cuda.synchronize()

    def fetch(self, adapters, stream):
        for a in adapters:
            self.pages[a] = slora.adapter_alloc(self.pool, a, int(self.w.ranks[a]), self.w.n_slots)
            self.host[a] = pinned_weights(self.w, a)
            slora.adapter_upload(self.pool, a, self.host[a].data_ptr(), stream.cuda_stream)

    def close(self):
        torch.cuda.synchronize()
        slora.pool_destroy(self.pool)


def apply(fp, ids, slot, stream=None):
    w = fp.w
    plan = slora.batch_plan(fp.pool, ids, None)
    x = bits_to_device(w.x_bits(slot), fp.dev)
    y = torch.from_numpy(w.y_in(slot)).to(fp.dev)
    slora.lora_apply(plan, slot, x.data_ptr(), y.data_ptr(), None if stream is None else stream.cuda_stream)
    return plan, x, y


def test_library_placed_adapters_fetched_from_pinned_memory():
    w = ragged_workload(801, synth.BF16, H=1000, n_pages=1200)
    fp = FetchedPool(w)
    side = torch.cuda.Stream()
    fp.fetch(range(w.n_adapters), side)
    side.synchronize()
    # pages: distinct, never a KV page; contents: bit for bit what the host holds
    allp = np.concatenate([p.reshape(-1) for p in fp.pages.values()])
    assert len(set(allp.tolist())) == allp.size and not set(allp.tolist()) & set(fp.kv.tolist())
    for a in range(w.n_adapters):
        r = int(w.ranks[a])
        if r == 0:
            continue
        for s in range(w.n_slots):
            for which in (0, 1):
                out = torch.empty((r, w.H), dtype=torch.int16, device=fp.dev)
                slora.adapter_gather(fp.pool, a, s, which, out.data_ptr())
                torch.cuda.synchronize()
                assert np.array_equal(out.cpu().numpy().view(np.uint16), w.weight_bits(a, s, which))
    pool = fp.pool_t.cpu().numpy().view(np.uint16)
    assert np.all(pool[fp.kv] == synth.nan_bits(w.dtype))                # KV pages were not written
    for slot in range(w.n_slots):
        plan, x, y = apply(fp, w.ids, slot)
        torch.cuda.synchronize()
        assert_close(y.cpu().numpy(), oracle_slot(w, slot), f"fetched pool, slot {slot}")
        slora.plan_destroy(plan)
    fp.close()


def test_fetch_on_a_side_stream_while_another_batch_computes():
    w = ragged_workload(802, synth.F16, H=1024, T=64, n_pages=1500)
    first = [a for a in range(w.n_adapters) if a % 2 == 0]
    later = [a for a in range(w.n_adapters) if a % 2 == 1]
    fp = FetchedPool(w)
    main, side = torch.cuda.Stream(), torch.cuda.Stream()
    fp.fetch(first, side)
    side.synchronize()
    ids_first = np.where(np.isin(w.ids, first), w.ids, -1).astype(np.int32)
    # the running batch uses the resident adapters while the others arrive on the side stream
    plan1, x1, y1 = apply(fp, ids_first, 0, main)
    fp.fetch(later, side)
    arrived = torch.cuda.Event()
    arrived.record(side)
    main.wait_event(arrived)                                             # the next batch needs them
    plan2, x2, y2 = apply(fp, w.ids, 0, main)
    main.synchronize()
    assert_close(y1.cpu().numpy(), oracle_slot(w, 0, ids=ids_first), "batch on resident adapters")
    assert_close(y2.cpu().numpy(), oracle_slot(w, 0), "batch after the fetch")
    slora.plan_destroy(plan1)
    slora.plan_destroy(plan2)
    fp.close()


def test_upload_rejects_pageable_memory_and_evicted_pages_are_reused():
    w = ragged_workload(803, synth.F16, H=256, n_pages=900)
    fp = FetchedPool(w)
    side = torch.cuda.Stream()
    a = int(np.argmax(w.ranks))
    fp.fetch([a], side)
    side.synchronize()
    pageable = np.zeros((w.n_slots, 2, int(w.ranks[a]), w.H), dtype=np.uint16)
    with pytest.raises(slora.SloraError) as e:
        slora.adapter_upload(fp.pool, a, pageable.ctypes.data, side.cuda_stream)
    assert e.value.code == slora.EINVAL
    free_before = slora.pool_free_pages(fp.pool)
    old = set(fp.pages[a].reshape(-1).tolist())
    slora.adapter_unload(fp.pool, a)                                     # eviction
    assert slora.pool_free_pages(fp.pool) == free_before + len(old)
    b = int(np.argsort(w.ranks)[-2])
    fp.fetch([b], side)
    side.synchronize()
    assert set(fp.pages[b].reshape(-1).tolist()) <= old                  # the released pages come back first
    ids = np.full(5, b, dtype=np.int32)
    wb = synth.make_workload("evict", 803, w.H, w.dtype, w.n_pages, w.n_slots, tuple(int(r) for r in w.ranks), ids)
    assert np.array_equal(wb.weight_bits(b, 0, 1), w.weight_bits(b, 0, 1))   # same seed: the same weights
    plan = slora.batch_plan(fp.pool, ids, None)
    x = bits_to_device(wb.x_bits(0), fp.dev)
    y = torch.from_numpy(wb.y_in(0)).to(fp.dev)
    slora.lora_apply(plan, 0, x.data_ptr(), y.data_ptr())
    torch.cuda.synchronize()
    assert_close(y.cpu().numpy(), oracle_slot(wb, 0), "adapter on reused pages")
    slora.plan_destroy(plan)
    fp.close()
