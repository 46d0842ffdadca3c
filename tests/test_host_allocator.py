"""The unified pool's page allocator on a host-only pool (no GPU needed): KV cache and adapters
draw from one set of free pages (Sec. 5.1), pages handed out are free and distinct, releases
are reusable, explicit page choices and library choices mix, and a failed request takes nothing."""
import numpy as np
import pytest

from paper_2311_03285_amd import slora
from paper_2311_03285_amd.slora import SloraError


def mk(n_pages=64, n_slots=2, max_rank=8):
    return slora.pool_init(256, n_pages, slora.F16, None, n_slots, max_rank)


def code(fn, *a, **k):
    with pytest.raises(SloraError) as e:
        fn(*a, **k)
    assert str(e.value)
    return e.value.code


def test_counts_follow_every_kind_of_ownership_change():
    p = mk()
    assert slora.pool_free_pages(p) == 64
    slora.pool_mark_kv(p, [3, 4, 5])
    assert slora.pool_free_pages(p) == 61
    slora.pool_mark_kv(p, [4, 5, 6])                     # 4, 5 already KV: only 6 is new
    assert slora.pool_free_pages(p) == 60
    slora.adapter_load(p, 0, 1, [10, 11, 12, 13])
    assert slora.pool_free_pages(p) == 56
    kv = slora.pool_alloc_kv(p, 7)
    assert slora.pool_free_pages(p) == 49
    pages = slora.adapter_alloc(p, 1, 2, 2)
    assert pages.shape == (2, 2, 2) and slora.pool_free_pages(p) == 41
    taken = set(kv.tolist()) | set(pages.reshape(-1).tolist())
    assert len(taken) == 15 and not taken & {3, 4, 5, 6, 10, 11, 12, 13}
    slora.adapter_unload(p, 0)
    slora.pool_mark_kv(p, kv, owned=False)
    slora.pool_mark_kv(p, [63], owned=False)             # already free: nothing changes
    assert slora.pool_free_pages(p) == 41 + 4 + 7
    slora.adapter_unload(p, 1)
    slora.pool_mark_kv(p, [3, 4, 5, 6], owned=False)
    assert slora.pool_free_pages(p) == 64
    slora.pool_destroy(p)


def test_kv_and_adapters_compete_and_a_failed_request_takes_nothing():
    p = mk(n_pages=40, n_slots=2, max_rank=8)
    kv = slora.pool_alloc_kv(p, 30)
    assert code(slora.adapter_alloc, p, 0, 4, 2) == slora.ENOMEM        # needs 16, 10 free
    assert slora.pool_free_pages(p) == 10
    assert code(slora.pool_alloc_kv, p, 11) == slora.ENOMEM
    assert slora.pool_free_pages(p) == 10
    slora.pool_mark_kv(p, kv[:6], owned=False)                          # the caller evicts KV pages
    pages = slora.adapter_alloc(p, 0, 4, 2)                             # and the same request succeeds
    assert slora.pool_free_pages(p) == 0
    assert not set(pages.reshape(-1).tolist()) & set(kv[6:].tolist())
    # the adapter is planned like any other
    plan = slora.batch_plan(p, [0, 0, -1], None)
    assert slora.plan_info(plan)["sum_rank"] == 4
    slora.plan_destroy(plan)
    slora.adapter_unload(p, 0)
    assert slora.pool_free_pages(p) == 16
    slora.pool_destroy(p)


def test_allocator_skips_pages_taken_by_index_after_their_release():
    p = mk(n_pages=16, n_slots=1, max_rank=4)
    a = slora.pool_alloc_kv(p, 16)
    slora.pool_mark_kv(p, a, owned=False)                # all 16 sit in the released stack
    slora.adapter_load(p, 5, 2, [0, 1, 2, 3])            # four of them are taken by index
    slora.pool_mark_kv(p, [8, 9])
    got = slora.pool_alloc_kv(p, 10)                     # everything that is left, each once
    assert sorted(got.tolist()) == [4, 5, 6, 7, 10, 11, 12, 13, 14, 15]
    assert code(slora.pool_alloc_kv, p, 1) == slora.ENOMEM
    slora.pool_destroy(p)


def test_adapter_alloc_argument_errors():
    p = mk()
    assert code(slora.adapter_alloc, p, -1, 1, 2) == slora.EINVAL
    assert code(slora.adapter_alloc, p, 0, 9, 2) == slora.ERANGE
    slora.adapter_alloc(p, 0, 1, 2)
    assert code(slora.adapter_alloc, p, 0, 1, 2) == slora.EBUSY          # already loaded
    assert slora.pool_free_pages(p) == 60
    assert slora.adapter_alloc(p, 1, 0, 2).size == 0                     # rank 0 takes no page
    assert code(slora.adapter_upload, p, 7, 0) == slora.ENOENT
    assert code(slora.adapter_upload, p, 0, 0) == slora.EHIP             # host-only pool
    assert code(slora.pool_alloc_kv, p, -1) == slora.EINVAL
    slora.pool_destroy(p)


def test_random_mix_keeps_ownership_consistent():
    g = np.random.default_rng(3)
    p = mk(n_pages=200, n_slots=2, max_rank=8)
    owner = {}                                           # page -> ("kv", None) | ("ad", id)
    adapters, kv_sets, next_id = {}, [], 0
    for _ in range(400):
        op = g.integers(0, 4)
        free = 200 - len(owner)
        assert slora.pool_free_pages(p) == free
        if op == 0:
            n = int(g.integers(0, 12))
            if n > free:
                assert code(slora.pool_alloc_kv, p, n) == slora.ENOMEM
                continue
            got = slora.pool_alloc_kv(p, n).tolist()
            assert len(set(got)) == n and not set(got) & set(owner)
            owner.update({q: ("kv", None) for q in got})
            kv_sets.append(got)
        elif op == 1:
            r = int(g.integers(0, 9))
            if 4 * r > free:
                assert code(slora.adapter_alloc, p, next_id, r, 2) == slora.ENOMEM
                continue
            got = slora.adapter_alloc(p, next_id, r, 2).reshape(-1).tolist()
            assert len(set(got)) == 4 * r and not set(got) & set(owner)
            owner.update({q: ("ad", next_id) for q in got})
            adapters[next_id] = got
            next_id += 1
        elif op == 2 and kv_sets:
            got = kv_sets.pop(int(g.integers(0, len(kv_sets))))
            slora.pool_mark_kv(p, got, owned=False)
            for q in got:
                del owner[q]
        elif op == 3 and adapters:
            i = list(adapters)[int(g.integers(0, len(adapters)))]
            slora.adapter_unload(p, i)
            for q in adapters.pop(i):
                del owner[q]
    slora.pool_destroy(p)
