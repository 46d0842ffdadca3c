"""Boundary validation and the scheduler, on a host-only pool (no GPU needed).

Every error must be reported before any state changes: after a failed call the pool accepts
the corrected call as if the failed one had never happened.
"""
import numpy as np
import pytest

from paper_2311_03285_amd import slora
from paper_2311_03285_amd.slora import SloraError


def mk(H=256, n_pages=64, n_slots=1, max_rank=16, dtype=slora.F16):
    return slora.pool_init(H, n_pages, dtype, None, n_slots, max_rank)


def code(fn, *a, **k):
    with pytest.raises(SloraError) as e:
        fn(*a, **k)
    assert str(e.value)                      # a message is always there
    return e.value.code


def test_pool_init_rejects_bad_shapes():
    for args in [(60, 8, 0), (257, 8, 0), (32776, 8, 0), (256, 0, 0), (256, 1 << 31, 0), (256, 8, 2)]:
        assert code(slora.pool_init, args[0], args[1], args[2], None, 1, 8) == slora.EINVAL
    assert code(slora.pool_init, 256, 8, 0, None, 0, 8) == slora.EINVAL
    assert code(slora.pool_init, 256, 8, 0, None, 1, 2000) == slora.EINVAL
    assert code(slora.pool_init, 256, 8, 0, 8, 1, 8) == slora.EINVAL     # misaligned device pointer


def test_adapter_load_validation_and_atomicity():
    p = mk()
    assert code(slora.adapter_load, p, -1, 1, [0, 1]) == slora.EINVAL
    assert code(slora.adapter_load, p, 0, -1, []) == slora.EINVAL
    assert code(slora.adapter_load, p, 0, 17, list(range(34))) == slora.ERANGE
    assert code(slora.adapter_load, p, 0, 2, [0, 1, 2]) == slora.EINVAL            # n_idx mismatch
    assert code(slora.adapter_load, p, 0, 2, [0, 1, 2, 64]) == slora.ERANGE
    assert code(slora.adapter_load, p, 0, 2, [0, 1, 2, -5]) == slora.ERANGE
    assert code(slora.adapter_load, p, 0, 2, [0, 1, 2, 1]) == slora.EBUSY          # repeated page
    # the failed calls left no marks: the same pages load fine now
    slora.adapter_load(p, 0, 2, [0, 1, 2, 3])
    assert code(slora.adapter_load, p, 0, 1, [8, 9]) == slora.EBUSY                # id taken
    assert code(slora.adapter_load, p, 1, 1, [3, 9]) == slora.EBUSY                # page of adapter 0
    slora.pool_mark_kv(p, [10, 11])
    assert code(slora.adapter_load, p, 1, 1, [9, 10]) == slora.EBUSY               # KV page
    slora.adapter_load(p, 1, 1, [9, 12])                                           # 9 was not left marked
    slora.adapter_load(p, 2, 0, [])                                                # rank 0 is legal
    slora.pool_destroy(p)


def test_kv_marking():
    p = mk()
    slora.adapter_load(p, 0, 1, [5, 6])
    assert code(slora.pool_mark_kv, p, [1, 64]) == slora.ERANGE
    assert code(slora.pool_mark_kv, p, [1, 5]) == slora.EBUSY
    assert code(slora.pool_mark_kv, p, [1, 2, 1]) == slora.EBUSY
    slora.adapter_load(p, 1, 1, [1, 2])          # pages 1, 2 were not left marked by the failures
    slora.pool_mark_kv(p, [3, 4])
    slora.pool_mark_kv(p, [3], owned=False)
    slora.adapter_load(p, 2, 1, [3, 7])
    assert code(slora.adapter_load, p, 3, 1, [4, 8]) == slora.EBUSY
    slora.pool_destroy(p)


def test_unload_frees_pages_and_stales_plans():
    p = mk()
    slora.adapter_load(p, 0, 2, [0, 1, 2, 3])
    plan = slora.batch_plan(p, [0, 0])
    assert code(slora.adapter_unload, p, 9) == slora.ENOENT
    slora.adapter_unload(p, 0)
    slora.adapter_load(p, 5, 2, [3, 2, 1, 0])
    assert code(slora.lora_apply, plan, 0, 16, 16) == slora.EBUSY           # stale plan
    assert code(slora.pool_destroy, p) == slora.EBUSY                       # live plan
    slora.plan_destroy(plan)
    slora.pool_destroy(p)


def test_multi_slot_list_length():
    p = mk(n_slots=3)
    assert code(slora.adapter_load, p, 0, 2, [0, 1, 2, 3]) == slora.EINVAL
    slora.adapter_load(p, 0, 2, list(range(12)))
    slora.pool_destroy(p)


def test_plan_validation():
    p = mk()
    slora.adapter_load(p, 0, 2, [0, 1, 2, 3])
    slora.adapter_load(p, 1, 1, [4, 5])
    assert code(slora.batch_plan, p, [0, 7]) == slora.ENOENT
    assert code(slora.batch_plan, p, [0, -2]) == slora.ENOENT
    assert code(slora.batch_plan, p, [0, 0, 1], [1, 2, 3]) == slora.ESEG          # does not start at 0
    assert code(slora.batch_plan, p, [0, 0, 1], [0, 2, 2, 3]) == slora.ESEG       # empty segment
    assert code(slora.batch_plan, p, [0, 0, 1], [0, 2]) == slora.ESEG             # does not end at T
    assert code(slora.batch_plan, p, [0, 0, 1], [0, 1000000, 3]) == slora.ESEG    # an offset far past T
    assert code(slora.batch_plan, p, [0, 1, 1], [0, 2, 3]) == slora.ESEG          # mixed ids in a segment
    plan = slora.batch_plan(p, [0, 0, 1], [0, 2, 3])
    assert code(slora.lora_apply, plan, 0, 16, 16) == slora.EHIP                  # host-only pool
    assert code(slora.lora_apply, plan, 1, 16, 16) == slora.ERANGE                # slot
    # the 16-bit-y entry points validate the same way
    assert code(slora.lora_apply_multi_y16, plan, [0], [16], [16]) == slora.EHIP
    assert code(slora.lora_apply_multi_y16, plan, [2], [16], [16]) == slora.ERANGE
    assert code(slora.lora_apply_multi_y16, plan, [0] * 9, [16] * 9, [16] * 9) == slora.EINVAL   # more than 8 slots
    assert code(slora.lora_expand_y16, plan, [0], [16]) == slora.EHIP
    slora.plan_destroy(plan)
    empty = slora.batch_plan(p, [])
    assert slora.plan_info(empty)["tokens"] == 0
    slora.plan_destroy(empty)
    slora.pool_destroy(p)


def test_scheduler_groups_buckets_and_routes():
    p = mk(H=1024, n_pages=4096, max_rank=64)
    at = 0
    ranks = {0: 8, 1: 64, 2: 16, 3: 0, 4: 64}
    for a, r in ranks.items():
        slora.adapter_load(p, a, r, np.arange(at, at + 2 * r))
        at += 2 * r
    slora.set_option(p, "mfma_min_tokens", 16)
    slora.set_option(p, "mfma_min_tiles", 1)
    ids = [0, 1, -1, 2, 3, 1, 0, 0] + [4] * 40
    seg = list(range(9)) + [48]
    plan = slora.batch_plan(p, ids, seg)
    info = slora.plan_info(plan)
    assert info["tokens"] == 3 + 2 + 1 + 40          # id -1 and the rank-0 adapter are dropped
    assert info["groups"] == 4
    assert info["groups_mfma"] == 1 and info["groups_vec"] == 3
    assert info["sum_rank"] == 8 + 64 + 16 + 64
    assert info["v_stride"] == 64
    # vector path, 4 pages per shrink item: adapter 1 (2 tokens, r=64): 16; adapter 2 (r=16): 4; adapter 0 (r=8): 2
    assert info["vec_shrink_items"] == 16 + 4 + 2
    assert info["vec_expand_items"] == 3 * (1024 // 512)
    assert info["mfma_shrink_items"] == 1             # 40 tokens: one item of two 32-token tiles
    assert info["mfma_expand_items"] == 2 * (1024 // 256)    # 40 tokens in tiles of 32
    slora.plan_destroy(plan)
    slora.set_option(p, "mfma_min_tokens", 1 << 40)
    plan = slora.batch_plan(p, ids, seg)
    assert slora.plan_info(plan)["groups_mfma"] == 0
    slora.plan_destroy(plan)
    slora.set_option(p, "mfma_min_tokens", 16)
    slora.set_option(p, "xcd_group", 3)
    assert code(slora.set_option, p, "xcd_group", 4) == slora.EINVAL
    plan = slora.batch_plan(p, ids, seg)
    grouped = slora.plan_info(plan)
    assert grouped["mfma_shrink_items"] == 1 and grouped["mfma_expand_items"] == 2 * (1024 // 256)
    slora.plan_destroy(plan)
    assert code(slora.set_option, p, "nope", 1) == slora.EINVAL
    assert code(slora.set_option, p, "mfma_min_tokens", 0) == slora.EINVAL
    # too few tiles to fill the GPU: the big group stays on the vector kernels
    slora.set_option(p, "mfma_min_tiles", 3)
    plan = slora.batch_plan(p, ids, seg)
    assert slora.plan_info(plan)["groups_mfma"] == 0
    slora.plan_destroy(plan)
    slora.pool_destroy(p)


def test_scheduler_shares_of_H_and_one_launch_decode_groups():
    """MFMA shrink tiles of 128 tokens x 128 ranks whose H range is handed to several workgroups,
    and the rule that sends decode groups to the one-launch kernel."""
    p = mk(H=4096, n_pages=1 << 15, max_rank=256, n_slots=4)
    at = 0
    for a, r in {0: 128, 1: 200, 2: 8}.items():
        slora.adapter_load(p, a, r, np.arange(at, at + 8 * r))
        at += 8 * r
    slora.set_option(p, "mfma_min_tiles", 1)
    slora.set_option(p, "mfma_split_bytes", 256 << 10)        # shares of about 256 KiB of rows
    ids = [0] * 300 + [1] * 130 + [2] * 20
    seg = [0, 300, 430, 450]
    plan = slora.batch_plan(p, ids, seg)
    info = slora.plan_info(plan)
    assert info["groups_mfma"] == 3 and info["v_stride"] == 224
    # tiles: adapter 0: 3 token tiles x 1 rank block; adapter 1: 2 x 2; adapter 2: 1 x 1
    whole = 3 + 4 + 1
    assert info["split_tiles"] >= 3 + 4 - 1 and info["mfma_shrink_items"] > whole
    assert info["mfma_expand_items"] == (10 + 5 + 1) * (4096 // 256)
    slora.plan_destroy(plan)
    slora.set_option(p, "mfma_split_bytes", 1 << 30)          # shares as large as any tile: nothing is split
    plan = slora.batch_plan(p, ids, seg)
    info = slora.plan_info(plan)
    assert info["split_tiles"] == 0 and info["mfma_shrink_items"] == whole
    slora.plan_destroy(plan)
    assert code(slora.set_option, p, "mfma_split_bytes", 100) == slora.EINVAL
    assert code(slora.set_option, p, "mfma_split_min_h", 64) == slora.EINVAL
    assert code(slora.set_option, p, "fuse_decode", 3) == slora.EINVAL
    assert code(slora.set_option, p, "shrink_pages", 0) == slora.EINVAL
    # decode groups: forced into the one-launch kernel, or not; never a group of more than 4 tokens
    dec = [0, 1, 2, 1, 0, 0, 0, 0]                            # adapter 0: five tokens
    for mode, want in ((0, 0), (1, 0), (2, 2)):
        slora.set_option(p, "fuse_decode", mode)
        plan = slora.batch_plan(p, dec)
        assert slora.plan_info(plan)["groups_fused"] == want, mode
        slora.plan_destroy(plan)
    slora.pool_destroy(p)
    # the default rule: enough small groups to fill the GPU, and large ones (>= 1 MiB of pages each)
    p = mk(H=8192, n_pages=1 << 17, max_rank=64, n_slots=8)
    for a in range(120):
        slora.adapter_load(p, a, 64, np.arange(a * 1024, (a + 1) * 1024))
    plan = slora.batch_plan(p, list(range(120)))              # 120 groups x 8 slots of 2 MiB each
    assert slora.plan_info(plan)["groups_fused"] == 120
    slora.plan_destroy(plan)
    plan = slora.batch_plan(p, list(range(60)))               # too few to fill the GPU
    assert slora.plan_info(plan)["groups_fused"] == 0
    slora.plan_destroy(plan)
    slora.pool_destroy(p)
