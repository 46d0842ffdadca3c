#!/usr/bin/env python3
"""Benchmark of the batched-LoRA hot path on one MI355X.

A step = one pass of the whole path (plan already built: shrink + expand for every projection
slot of the workload) over one batch of synthetic input that is resident in HBM.  Steps rotate
over several distinct batches drawn against the same resident adapters, so consecutive steps
do not find their pages in the caches.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 4] [--law power|zipf]
                    [--batches R] [--mode fused|qkv_o|per_slot] [--no-cpu]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
# HBM bytes per launch of a stage from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, each scaled by what
# the counter reads for the library's plain page-copy kernel of known size: FETCH_SIZE / factor +
# WRITE_SIZE, summed over the kernels of the stage (the MFMA shrink counts with its join kernel).
# From the committed counter summaries named in "source"; only for the default command lines of
# these workloads with fp32 y.  On cfg5 the figures are those of the two-stage kernels the
# per-stage timing loop launches (a whole apply runs the decode groups in one kernel instead).
MEASURED_TRAFFIC = {("cfg4-large-pool-decode", "power", "fused", 8): {"expand_vec": 332880461,
                                                                        "shrink_vec": 312123908,
                                                                        "source": "profiles/cfg4_decode_hbm_traffic.md"},
                    ("cfg3-prefill", "power", "fused", 8): {"expand_mfma": 690047714,
                                                            "shrink_mfma": 209097830 + 7899366,
                                                            "source": "profiles/cfg3_prefill_hbm_traffic.md"},
                    ("cfg5-mixed", "power", "fused", 8): {"expand_vec+mfma": 2804682598 + 1373456197,
                                                          "shrink_vec+mfma": 768431054 + 36335013 + 1299029045,
                                                          "source": "profiles/cfg5_mixed_hbm_traffic.md"}}
MFMA_PEAK_TFLOPS = 2500.0      # dense fp16 / bf16 MFMA, published


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def measure(args, workload: int, no_cpu: bool) -> dict:
    """Time one workload; returns the JSON object of its bench line."""
    import torch
    from paper_2311_03285_amd import slora, synth
    from paper_2311_03285_amd.harness import DeviceWorkload, bits_to_device

    if not torch.cuda.is_available():
        raise RuntimeError("no GPU visible")
    slora.lib()                                   # fail loudly if the HIP library is missing
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    t_setup = time.time()
    R = max(1, args.batches)
    wls = [synth.config(workload, batch=b, law=args.law) for b in range(R)]
    w0 = wls[0]
    n_slots = w0.n_slots
    # the pool: every adapter loaded at its scattered pages; seeded weights for the adapters of
    # batch 0 (the oracle's sample uses them), finite filler for the rest, NaN on KV pages
    dw = DeviceWorkload(w0, device=dev, real_adapters="used", slots=list(range(n_slots)), threads=16)
    log(f"[bench] pool ready: {w0.name}, {w0.n_pages} pages x {w0.H} ({w0.n_pages * w0.H * 2 / 1e9:.1f} GB), "
        f"{w0.n_adapters} adapters, {n_slots} slots, setup {time.time() - t_setup:.1f}s")

    for kv in args.opt:
        k, v = kv.split("=")
        slora.set_option(dw.pool, k, int(v))
    stream = torch.cuda.Stream(device=dev)
    plans, xs, ys = [], [], []
    for b, w in enumerate(wls):
        plans.append(dw.plan(ids=w.ids, seg_offsets=w.seg_offsets))
        # one activation buffer per projection (q, k, v would share theirs in a model; separate
        # buffers keep cache hits on x from flattering the byte rate) and one y per slot
        xs.append([bits_to_device(w.x_bits(s), dev) for s in range(min(n_slots, 4))])
        if args.y16:    # y in the pool's 16-bit storage type
            ys.append([bits_to_device(w.y16_bits(s % 4), dev) for s in range(n_slots)])
        else:
            ys.append([torch.from_numpy(w.y_in(s % 4)).to(dev) for s in range(n_slots)])
    torch.cuda.synchronize()
    # plan time on an idle device: host scheduler + work-list upload, per batch
    plan_s = []
    for w in wls:
        tp = time.perf_counter()
        extra = slora.batch_plan(dw.pool, w.ids, w.seg_offsets)
        plan_s.append(time.perf_counter() - tp)
        slora.plan_destroy(extra)
    info = slora.plan_info(plans[0])
    log(f"[bench] plan[0]: {info}")

    slots = list(range(n_slots))

    def x_of(b, s):
        # --shared-x: the q, k and v projections of a layer (slots 4l .. 4l+2) read one buffer
        return xs[b][3 if s % 4 == 3 else 0].data_ptr() if args.shared_x else xs[b][s % 4].data_ptr()

    apply_multi = slora.lora_apply_multi_y16 if args.y16 else slora.lora_apply_multi
    expand = slora.lora_expand_y16 if args.y16 else slora.lora_expand
    apply_one = lambda p, s, x, y, st: apply_multi(p, [s], [x], [y], st)

    def step(b):
        p = plans[b]
        if args.mode == "fused":
            for g0 in range(0, n_slots, slora.MAX_MULTI):
                g = slots[g0:g0 + slora.MAX_MULTI]
                apply_multi(p, g, [x_of(b, s) for s in g], [ys[b][s].data_ptr() for s in g], stream)
        elif args.mode == "qkv_o":
            for l0 in range(0, n_slots, 4):
                g = slots[l0:l0 + 3]
                apply_multi(p, g, [x_of(b, s) for s in g], [ys[b][s].data_ptr() for s in g], stream)
                for s in slots[l0 + 3:l0 + 4]:
                    apply_one(p, s, x_of(b, s), ys[b][s].data_ptr(), stream)
        else:
            for s in slots:
                apply_one(p, s, x_of(b, s), ys[b][s].data_ptr(), stream)

    # ---- set-up: every rotating batch is applied once, so that each plan owns its v scratch
    # (the first apply of a plan allocates it) whatever the number of warm-up steps -----------
    # and the device is kept busy for a while: after the host-side set-up it has been idle for
    # seconds, and the first milliseconds of work after that run below the steady-state rate.
    spin = []
    t_spin = time.perf_counter()
    while len(spin) < 2 or (time.perf_counter() - t_spin < args.spin_ms * 1e-3 and len(spin) < 10000):
        ta = time.perf_counter()
        for b in range(R):
            step(b)
        torch.cuda.synchronize()
        spin.append((time.perf_counter() - ta) * 1e3 / R)
    log(f"[bench] set-up rotations, ms per step: first {spin[0]:.4f}, second {spin[1]:.4f}, last {spin[-1]:.4f} ({len(spin)} rotations)")
    # ---- timed region: W warm-up steps, then K steps, inputs resident -----------------------
    for i in range(args.warmup):
        step(i % R)
    torch.cuda.synchronize()
    graph = None
    if args.graph:
        # one HIP graph holding a full rotation of R steps (apply makes no allocation once the
        # plans' scratch exists); K is rounded down to a multiple of R
        graph = torch.cuda.CUDAGraph()
        real_stream = stream
        with torch.cuda.graph(graph, stream=real_stream):
            stream = torch.cuda.current_stream()
            for b in range(R):
                step(b)
        stream = real_stream
        graph.replay()
        torch.cuda.synchronize()
        args.steps = max(R, args.steps // R * R)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    if graph is None:
        e0.record(stream)
        for i in range(args.steps):
            step(i % R)
        e1.record(stream)
    else:
        with torch.cuda.stream(stream):
            e0.record(stream)
            for i in range(args.steps // R):
                graph.replay()
            e1.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ev_ms = e0.elapsed_time(e1)
    ms_per_step = wall * 1e3 / args.steps

    def per_step_ms(batches, n):
        """Each step bracketed by its own pair of events: (median, min) in ms."""
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
        ev[0].record(stream)
        for i in range(n):
            step(batches[i % len(batches)])
            ev[i + 1].record(stream)
        torch.cuda.synchronize()
        d = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(n))
        return d[n // 2], d[0]

    # ---- the per-batch life-cycle (Sec. 4.1: a new batch every iteration) ---------------------
    # (a) plan + apply of every slot + plan_destroy per step, nothing waited for in between;
    # (b) the one-shot call (plan + apply of ONE slot + destroy) back to back.  Wall clock per
    # cycle including the final synchronisation, and the host's share of it (time until the
    # calls of a cycle have returned).
    def cycle(b):
        p = slora.batch_plan(dw.pool, wls[b].ids, wls[b].seg_offsets)
        for g0 in range(0, n_slots, slora.MAX_MULTI):
            g = slots[g0:g0 + slora.MAX_MULTI]
            apply_multi(p, g, [x_of(b, s) for s in g], [ys[b][s].data_ptr() for s in g], stream)
        slora.plan_destroy(p)

    def one_shot(b):
        if args.y16:
            return
        slora.lora_shrink_expand(dw.pool, 0, x_of(b, 0), wls[b].ids, wls[b].seg_offsets, ys[b][0].data_ptr(), stream)

    def timed_calls(fn, n):
        for i in range(2 * R):
            fn(i % R)
        torch.cuda.synchronize()
        t_a = time.perf_counter()
        for i in range(n):
            fn(i % R)
        t_b = time.perf_counter()
        torch.cuda.synchronize()
        t_c = time.perf_counter()
        return (t_c - t_a) * 1e3 / n, (t_b - t_a) * 1e3 / n

    n_cyc = max(R, min(args.steps, 64))
    cyc_ms, cyc_host_ms = timed_calls(cycle, n_cyc)
    shot_ms, shot_host_ms = timed_calls(one_shot, n_cyc) if not args.y16 else (None, None)
    stats_a = slora.pool_stats(dw.pool)
    timed_calls(cycle, R)
    stats_b = slora.pool_stats(dw.pool)

    cold_med, cold_min = per_step_ms(list(range(R)), max(R, min(args.steps, 64)))
    per_step_ms([0], 8)
    warm_med, warm_min = per_step_ms([0], 32)       # the same batch again and again: caches help
    # what two dependent, near-empty launches cost on this stream (one-element torch kernels, back
    # to back like the steps): the floor under a step made of a shrink and an expand launch
    tiny = torch.zeros(1, device=dev)
    with torch.cuda.stream(stream):
        for _ in range(20):
            tiny.add_(1.0)
        f0, f1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        f0.record(stream)
        for _ in range(200):
            tiny.add_(1.0)
            tiny.add_(1.0)
        f1.record(stream)
    torch.cuda.synchronize()
    launch_floor_us = f0.elapsed_time(f1) * 1e3 / 200
    # The K timed steps visit batch i % R: when K is no multiple of R the batches (which differ in
    # size) are not visited equally often, so tokens, bytes and flops per step are averaged with
    # the weights of the steps that were timed.
    mix = np.bincount([i % R for i in range(args.steps)], minlength=R) / float(args.steps)
    avg = lambda f, wts=mix: float(np.dot(wts, [float(f(w)) for w in wls]))

    def step_bytes(wts):
        b = avg(lambda w: w.algorithmic_bytes(), wts) * n_slots
        if args.y16:        # y read + written as 2-byte elements instead of 4-byte ones
            b -= 2 * avg(lambda w: np.count_nonzero(w.ids >= 0) * w.H, wts) * 2 * n_slots
        if args.shared_x:
            # x of a layer's q, k, v counted once: two of every four slots' x reads drop out
            b -= avg(lambda w: np.count_nonzero(w.ids >= 0) * w.H * 2, wts) * sum(1 for s in range(n_slots) if s % 4 in (1, 2))
        return b

    tok_per_step = avg(lambda w: w.T)
    bytes_step = step_bytes(mix)
    bytes_step_even = step_bytes(np.full(R, 1.0 / R))      # for the per-step brackets, which cycle evenly
    t_act_b = float(np.mean([np.count_nonzero(w.ids >= 0) * w.H for w in wls]))
    flops_step = avg(lambda w: w.flops()) * n_slots
    # the same traffic if every token fetched its adapter's pages for itself (no sharing)
    naive_step = avg(lambda w: int(2 * w.ranks[w.ids[w.ids >= 0]].astype(np.int64).sum()) * w.H * 2 +
                     np.count_nonzero(w.ids >= 0) * w.H * (2 + 8)) * n_slots
    value = tok_per_step * args.steps / wall

    # ---- per-kernel durations: HIP events on the launch stream around runs of one stage ----------
    # (the shrink of every rotating batch back to back, then the expand of every batch: each plan
    # keeps its own v, and no event record sits between two launches of a run)
    def stage_times(n_rounds):
        sh, ex = [], []
        for _ in range(n_rounds):
            for g0 in range(0, n_slots, slora.MAX_MULTI):
                g = slots[g0:g0 + slora.MAX_MULTI]
                ea, eb, ec = (torch.cuda.Event(enable_timing=True) for _ in range(3))
                ea.record(stream)
                for b in range(R):
                    slora.lora_shrink(plans[b], g, [x_of(b, s) for s in g], stream)
                eb.record(stream)
                for b in range(R):
                    expand(plans[b], g, [ys[b][s].data_ptr() for s in g], stream)
                ec.record(stream)
                sh.append((ea, eb, len(g)))
                ex.append((eb, ec, len(g)))
        torch.cuda.synchronize()
        f = lambda L: [(a.elapsed_time(b_) * 1e-3 / R, n) for a, b_, n in L]
        return f(sh), f(ex)

    stage_times(2)
    sh, ex = stage_times(max(2, min(args.steps // R, 16)))
    sh_b = float(np.mean([w.shrink_bytes() for w in wls]))
    ex_b = float(np.mean([w.expand_bytes() for w in wls]))
    if args.y16:
        ex_b -= 2 * t_act_b * 2
    sh_t = float(np.mean([t for t, n in sh]))
    ex_t = float(np.mean([t for t, n in ex]))
    if args.shared_x:
        # per slot of a launch: the x bytes of q, k, v are counted once (2 distinct buffers per 4 slots)
        x_b = float(np.mean([np.count_nonzero(w.ids >= 0) * w.H * 2 for w in wls]))
        sh_b -= x_b / 2
    sh_gbs = float(np.mean([sh_b * n / t for t, n in sh])) / 1e9
    ex_gbs = float(np.mean([ex_b * n / t for t, n in ex])) / 1e9
    dom = "expand" if ex_t >= sh_t else "shrink"
    dom_gbs = ex_gbs if dom == "expand" else sh_gbs
    kinds = ("mfma" if info["groups_mfma"] and not info["groups_vec"] else
             "vec" if not info["groups_mfma"] else "vec+mfma")
    traffic = ({} if args.y16 or args.shared_x or args.opt else
               MEASURED_TRAFFIC.get((w0.name, args.law, args.mode, R), {}))
    roofline = {
        "bound": "hbm", "kernel": f"{dom}_{kinds}", "achieved": round(dom_gbs, 1), "peak": HBM_PEAK_GBS,
        "unit": "GB/s", "frac": round(dom_gbs / HBM_PEAK_GBS, 4),
        "traffic": traffic.get(f"{dom}_{kinds}"),
        # counters cannot be read inside a timed run: the figure comes from the committed summary
        "traffic_source": (None if not traffic else f"{traffic['source']} (earlier rocprofv3 --pmc runs of this command)"),
        "algorithmic_bytes_per_launch": int((ex_b if dom == "expand" else sh_b) * min(n_slots, slora.MAX_MULTI)),
        "avg_launch_us": round((ex_t if dom == "expand" else sh_t) * 1e6, 2),
        "other_kernel": {"kernel": f"{'shrink' if dom == 'expand' else 'expand'}_{kinds}",
                         "achieved": round(sh_gbs if dom == "expand" else ex_gbs, 1),
                         "avg_launch_us": round((sh_t if dom == "expand" else ex_t) * 1e6, 2)},
        "slots_per_launch": min(n_slots, slora.MAX_MULTI),
    }

    # ---- parity of the timed launch shape: batch 0, EVERY slot, against the oracle -----------------
    # The GPU side is the call the timed loop makes (all slots, up to 8 per launch pair, on the
    # plan of batch 0) on fresh y buffers.  The oracle computes a seeded sample of the tokens one
    # by one (all of them when the batch is small); sampled rows are compared element by element.
    from oracle import c_oracle
    w = w0
    act = np.nonzero(w.ids >= 0)[0]
    n_samp = int(min(act.size, args.parity_tokens))
    samp = np.sort(np.random.default_rng(w.seed).choice(act, size=n_samp, replace=False)) if n_samp else act
    ids_s = np.full_like(w.ids, -1)
    ids_s[samp] = w.ids[samp]
    samp_d = torch.from_numpy(samp).to(dev)
    rel = mx = 0.0
    for g0 in range(0, n_slots, slora.MAX_MULTI):
        grp = slots[g0:g0 + slora.MAX_MULTI]
        yg = [torch.from_numpy(w.y_in(s % 4)).to(dev) for s in grp]
        slora.lora_apply_multi(plans[0], grp, [x_of(0, s) for s in grp], [t.data_ptr() for t in yg], stream)
        torch.cuda.synchronize()
        for s, t in zip(grp, yg):
            if not n_samp:
                continue
            rows, lists = w.compact_pool(s, np.unique(ids_s[samp]))
            xb = w.x_bits((3 if s % 4 == 3 else 0) if args.shared_x else s % 4)
            ref = c_oracle.lora_apply(rows, w.dtype, lists, ids_s, xb, w.y_in(s % 4))[samp]
            got = t[samp_d].cpu().numpy().astype(np.float64)
            rel = max(rel, float(np.linalg.norm(got - ref) / np.linalg.norm(ref)))
            mx = max(mx, float(np.abs(got - ref).max()))
        del yg
    parity = {"slots_checked": n_slots, "tokens_checked_per_slot": n_samp, "of_tokens": int(act.size),
              "rel_l2": float(f"{rel:.3e}"), "max_abs": float(f"{mx:.3e}"), "bars": {"rel_l2": 1e-3, "max_abs": 1e-2}}
    if not (np.isfinite(rel) and rel <= 1e-3 and mx <= 1e-2):
        raise RuntimeError(f"GPU result disagrees with the oracle (rel-L2 {rel:.3e}, max-abs {mx:.3e})")

    # ---- the oracle as it stands, timed on this machine's host cores ---------------------------------
    cpu = None
    if not no_cpu:
        packs = [(s, w.compact_pool(s), w.x_bits(s), w.y_in(s)) for s in range(min(n_slots, 4))]
        _, cores = c_oracle.lora_apply(packs[0][1][0], w.dtype, packs[0][1][1], w.ids[:1], packs[0][2][:1],
                                       packs[0][3][:1], return_threads=True)
        # timing: whole passes (all tokens of batch 0 x the seeded slots) until ~cpu_seconds of
        # summed core time have been spent
        passes, t_cpu = 0, 0.0
        while t_cpu * cores < args.cpu_seconds and passes < 1000:
            tc = time.perf_counter()
            for s, (rows, lists), xb, yb in packs:
                c_oracle.lora_apply(rows, w.dtype, lists, w.ids, xb, yb)
            t_cpu += time.perf_counter() - tc
            passes += 1
        # one thread, a bounded sample: the first tokens of batch 0 on the first seeded slot
        s1, (rows1, lists1), xb1, yb1 = packs[0]
        k1 = int(min(w.T, 32))
        tc = time.perf_counter()
        c_oracle.lora_apply(rows1, w.dtype, lists1, w.ids[:k1], xb1[:k1], yb1[:k1], n_threads=1)
        t_one = time.perf_counter() - tc
        pairs = passes * len(packs) * w.T                       # (token, slot) units done
        cpu = {"value": round(pairs / t_cpu / n_slots, 2), "unit": "tokens/s", "cores": int(cores),
               "kind": "oracle",
               "sample": f"{passes} pass(es) over the {w.T} tokens of batch 0 x {len(packs)} slot(s): "
                         f"{t_cpu:.2f}s wall on {cores} threads, scaled to the {n_slots} slots a token "
                         "passes per step; the oracle reads a compact re-paging of the adapters batch 0 "
                         "uses (same weights, pages renumbered), not the full-size pool",
               "value_1_thread": round(k1 / t_one / n_slots, 2),
               "sample_1_thread": f"{k1} tokens x 1 slot in {t_one:.2f}s on 1 thread, scaled the same way"}

    fetch = None
    if args.fetch:
        # adapters of waiting requests arriving from pinned host memory on a side stream while the
        # steps run (Sec. 5.2): step time alone / under the fetch, fetch rate alone / under the steps
        rank, n_new = 64, args.fetch
        per_adapter = w0.n_slots * 2 * rank
        free = np.ones(w0.n_pages, dtype=bool)
        free[w0.owned_pages()] = False
        give = np.nonzero(free)[0][:n_new * per_adapter].astype(np.int32)      # KV pages handed back
        slora.pool_mark_kv(dw.pool, give, False)
        host = (torch.randn((n_new, per_adapter, w0.H)) * 0.02).to(torch.float16).view(torch.int16).pin_memory()
        new_ids = [w0.n_adapters + 1000 + i for i in range(n_new)]
        for a in new_ids:
            slora.adapter_alloc(dw.pool, a, rank, w0.n_slots)
        side = torch.cuda.Stream(device=dev)
        fetch_bytes = n_new * per_adapter * w0.H * 2

        def fetch_all():
            for i, a in enumerate(new_ids):
                slora.adapter_upload(dw.pool, a, host[i].data_ptr(), side)

        def timed(do_steps, do_fetch, reps=3):
            best_s, best_f = None, None
            for _ in range(reps):
                s0, s1, f0, f1 = (torch.cuda.Event(enable_timing=True) for _ in range(4))
                torch.cuda.synchronize()
                n_steps = 8 * R
                s0.record(stream)
                if do_steps:            # enqueued first: the GPU is busy with them while the host
                    for i in range(n_steps):        # issues the uploads
                        step(i % R)
                s1.record(stream)
                f0.record(side)
                if do_fetch:
                    fetch_all()
                f1.record(side)
                torch.cuda.synchronize()
                ts, tf = s0.elapsed_time(s1) / n_steps, f0.elapsed_time(f1)
                best_s = ts if best_s is None else min(best_s, ts)
                best_f = tf if best_f is None else min(best_f, tf)
            return best_s, best_f

        timed(True, True, 1)
        s_alone, _ = timed(True, False)
        _, f_alone = timed(False, True)
        s_both, f_both = timed(True, True)
        fetch = {"adapters": n_new, "rank": rank, "bytes": fetch_bytes,
                 "fetch_ms_alone": round(f_alone, 4), "fetch_gbps_alone": round(fetch_bytes / f_alone / 1e6, 1),
                 "fetch_ms_under_compute": round(f_both, 4),
                 "step_ms_alone": round(s_alone, 5), "step_ms_under_fetch": round(s_both, 5)}

    # what a plain streaming copy reaches on this machine (torch's elementwise copy of 1 GiB: read +
    # write), as a measured companion to the nominal 8 TB/s
    a_ = torch.empty(1 << 30, dtype=torch.int8, device=dev)
    b_ = torch.empty_like(a_)
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    with torch.cuda.stream(stream):
        b_.copy_(a_)
        c0.record(stream)
        for _ in range(5):
            b_.copy_(a_)
        c1.record(stream)
    torch.cuda.synchronize()
    copy_gbs = 5 * 2 * a_.numel() / (c0.elapsed_time(c1) * 1e-3) / 1e9
    del a_, b_
    # and what the library GEMM (hipBLASLt through torch) reaches on an 8192^3 product in the
    # storage type, as a measured companion to the nominal dense MFMA peak
    tdt_ = torch.float16 if w0.dtype == 0 else torch.bfloat16
    ga = (torch.randn((8192, 8192), device=dev) * 0.01).to(tdt_)
    gb = (torch.randn((8192, 8192), device=dev) * 0.01).to(tdt_)
    gc = torch.empty((8192, 8192), dtype=tdt_, device=dev)
    with torch.cuda.stream(stream):
        torch.matmul(ga, gb, out=gc)
        c0.record(stream)
        for _ in range(5):
            torch.matmul(ga, gb, out=gc)
        c1.record(stream)
    torch.cuda.synchronize()
    gemm_tflops = 5 * 2 * 8192 ** 3 / (c0.elapsed_time(c1) * 1e-3) / 1e12
    del ga, gb, gc
    roofline["measured_gemm_tflops"] = round(gemm_tflops, 1)
    roofline["measured_copy_gbps"] = round(copy_gbs, 1)
    roofline["frac_of_measured_copy"] = round(dom_gbs / copy_gbs, 4)

    ablation = None
    plain = args.mode == "fused" and not (args.y16 or args.graph or args.shared_x or args.opt)
    if args.ablation == "on" or (args.ablation == "auto" and plain and workload in (3, 4)):
        # (1) the padded batched-matmul formulation the paper compares its kernels with
        #     (Sec. 7.1, "bmm"): gather every token's adapter from the pool into contiguous
        #     tensors padded to the largest rank, then two torch.bmm calls; (2) the base
        #     projection x W on a second stream while the LoRA step runs (Fig. 1: the two are
        #     independent until the add).  Library GEMMs only; slot 0 of batch 0.
        tdt = torch.float16 if w0.dtype == 0 else torch.bfloat16
        pool16 = dw.pool_t.view(tdt)
        free = np.ones(w0.n_pages, dtype=bool)
        free[w0.owned_pages()] = False
        zero_page = int(np.nonzero(free)[0][0])                  # a KV page of this bench's pool
        slora.pool_write_pages(dw.pool, [zero_page], np.zeros((1, w0.H), np.uint16), False)
        act = np.nonzero(w0.ids >= 0)[0]
        rmax = int(w0.ranks[w0.ids[act]].max())
        ia = np.full((act.size, rmax), zero_page, dtype=np.int64)
        ib = np.full((act.size, rmax), zero_page, dtype=np.int64)
        for k, t in enumerate(act):
            pg = w0.page_idx[int(w0.ids[t])][0]
            ia[k, :pg.shape[1]] = pg[0]
            ib[k, :pg.shape[1]] = pg[1]
        ia_d, ib_d = torch.from_numpy(ia).to(dev), torch.from_numpy(ib).to(dev)
        act_d = torch.from_numpy(act).to(dev)
        x16 = xs[0][0].view(tdt)
        y32 = ys[0][0].float() if args.y16 else ys[0][0].clone()

        def bmm_step():
            At = pool16[ia_d]                                       # [T, rmax, H]: rows = columns of A
            Bm = pool16[ib_d]                                       # [T, rmax, H]
            xv = x16[act_d].unsqueeze(1)                            # [T, 1, H]
            v = torch.bmm(xv, At.transpose(1, 2))                   # [T, 1, rmax]
            y32[act_d] += torch.bmm(v, Bm).squeeze(1).float()

        def time_on(st, fn, reps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            with torch.cuda.stream(st):
                fn()
                torch.cuda.synchronize()
                a.record(st)
                for _ in range(reps):
                    fn()
                b.record(st)
            torch.cuda.synchronize()
            return a.elapsed_time(b) / reps

        # the two formulations against each other on the same fresh y (the delta they add)
        y_in0 = torch.from_numpy(w0.y_in(0)).to(dev)
        with torch.cuda.stream(stream):
            y32.copy_(y_in0)
            bmm_step()
            d_bmm = (y32 - y_in0).double()
            y_k = y_in0.clone()
            slora.lora_apply(plans[0], 0, x_of(0, 0), y_k.data_ptr(), stream)
            d_ker = (y_k - y_in0).double()
            bmm_vs_kernels = float((d_bmm - d_ker).norm() / d_ker.norm())
        del y_in0, y_k, d_bmm, d_ker
        t_bmm = time_on(stream, bmm_step, 5)
        one_slot = lambda: apply_one(plans[0], 0, x_of(0, 0), ys[0][0].data_ptr(), stream)
        t_ours = time_on(stream, one_slot, 20)
        # base projection of the whole batch on a second stream
        W = (torch.randn((w0.H, w0.H), device=dev) * 0.02).to(tdt)
        xw = torch.empty((x16.shape[0], w0.H), dtype=tdt, device=dev)
        side = torch.cuda.Stream(device=dev)
        gemm = lambda: torch.matmul(x16, W, out=xw)
        t_gemm = time_on(side, lambda: [gemm() for _ in range(n_slots)], 20)
        t_step = time_on(stream, lambda: step(0), 20)
        a0, a1, g1 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
        torch.cuda.synchronize()
        a0.record(stream)
        side.wait_event(a0)
        for _ in range(20):
            step(0)
            with torch.cuda.stream(side):
                for _ in range(n_slots):
                    gemm()
        a1.record(stream)
        g1.record(side)
        torch.cuda.synchronize()
        t_both = max(a0.elapsed_time(a1), a0.elapsed_time(g1)) / 20
        ablation = {"padded_bmm_ms_per_slot": round(t_bmm, 4), "lora_kernels_ms_per_slot": round(t_ours, 4),
                    "padded_bmm_rank": rmax, "speedup_over_padded_bmm": round(t_bmm / t_ours, 2),
                    # the bmm's v and output are rounded to the 16-bit type: agreement to ~1e-3
                    "padded_bmm_vs_lora_kernels_rel_l2_of_delta": bmm_vs_kernels,
                    "base_gemm_ms_per_step": round(t_gemm, 4), "lora_ms_per_step": round(t_step, 4),
                    "both_streams_ms_per_step": round(t_both, 4),
                    "serial_ms_per_step": round(t_gemm + t_step, 4)}

    out = {
        "metric": "lora_tokens_per_s", "value": round(value, 1), "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": w0.name, "H": w0.H, "storage": "fp16" if w0.dtype == 0 else "bf16",
                   "adapters": w0.n_adapters, "tokens_per_step": tok_per_step, "slots": n_slots,
                   "pool_pages": w0.n_pages, "popularity": args.law, "rotating_batches": R,
                   "launch_mode": args.mode + ("+hipgraph" if args.graph else "") + ("+shared_x" if args.shared_x else "") + ("+y16" if args.y16 else ""),
                   "distinct_adapters_per_batch": float(np.mean([len(w.used_adapters()) for w in wls]))},
        "hbm_gbps": round(bytes_step / (wall / args.steps) / 1e9, 1),
        "hbm_frac": round(bytes_step / (wall / args.steps) / 1e9 / HBM_PEAK_GBS, 4),
        "hbm_frac_median_step": round(bytes_step_even / (cold_med * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        "mfma_util": round(flops_step / (wall / args.steps) / 1e12 / MFMA_PEAK_TFLOPS, 5),
        # the most the matrix cores can be busy while HBM keeps up: arithmetic intensity x 8 TB/s
        "mfma_util_cap": round(flops_step / bytes_step * HBM_PEAK_GBS * 1e9 / (MFMA_PEAK_TFLOPS * 1e12), 5),
        "algorithmic_bytes_per_step": int(bytes_step), "flops_per_step": int(flops_step),
        "event_ms_per_step": round(ev_ms / args.steps, 5),
        "step_ms_median": round(cold_med, 5), "step_ms_min": round(cold_min, 5),
        "warm_step_ms_median": round(warm_med, 5), "warm_step_ms_min": round(warm_min, 5),
        "plan_ms": round(float(np.median(plan_s)) * 1e3, 4),
        # a new plan every step: plan + apply of all slots + plan_destroy, pipelined (wall per
        # cycle with the final synchronisation; host = until the cycle's calls have returned)
        "plan_lifecycle_ms": round(cyc_ms, 5), "plan_lifecycle_host_ms": round(cyc_host_ms, 5),
        "plan_lifecycle_over_apply_ms": round(cyc_ms - ms_per_step, 5),
        "one_shot_ms": None if shot_ms is None else round(shot_ms, 5),
        "one_shot_host_ms": None if shot_ms is None else round(shot_host_ms, 5),
        "allocations_in_steady_cycles": stats_b["allocations"] - stats_a["allocations"],
        "launch_floor_us": round(launch_floor_us, 2),
        "naive_bytes_per_step": int(naive_step),
        "roofline": roofline, "cpu_baseline": cpu, "parity": parity,
    }
    if fetch:
        out["fetch"] = fetch
    if ablation:
        out["ablation"] = ablation
    dw.close()
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", type=int, default=4, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--law", default="power", choices=["power", "zipf"])
    ap.add_argument("--batches", type=int, default=8, help="distinct batches the steps rotate over")
    ap.add_argument("--mode", default="fused", choices=["fused", "qkv_o", "per_slot"])
    ap.add_argument("--ablation", default="auto", choices=["auto", "on", "off"],
                    help="also time the padded torch.bmm formulation of one slot and the base projection "
                         "x W running on a second stream beside the LoRA step (auto: for the plain fused runs "
                         "of workloads 3 and 4)")
    ap.add_argument("--fetch", type=int, default=0,
                    help="also time the upload of this many rank-64 adapters from pinned host memory on a side "
                         "stream, alone and while the steps run")
    ap.add_argument("--y16", action="store_true",
                    help="y in the pool's 16-bit storage type (rounded once at the store) instead of fp32")
    ap.add_argument("--shared-x", action="store_true",
                    help="q, k, v of a layer read the same x buffer (as in a model); its bytes are counted once")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--graph", action="store_true", help="replay the steps as one HIP graph per rotation")
    ap.add_argument("--spin-ms", type=float, default=50.0,
                    help="untimed set-up: rotations over the batches until this much time has passed (at least two)")
    ap.add_argument("--opt", action="append", default=[], help="library tuning option key=value (repeatable)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="core-seconds of oracle work to time")
    ap.add_argument("--parity-tokens", type=int, default=32,
                    help="tokens per slot of batch 0 the oracle recomputes for the in-run parity check")
    ap.add_argument("--also", default="2,3,5", help="workloads whose summary is nested under 'also' when the "
                    "primary one is config 4 (comma list, 'none' to skip)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
              "run it with --gpus 1", file=sys.stderr)
        return 2

    try:
        out = measure(args, args.workload, args.no_cpu)
        if args.workload == 4 and args.also != "none":
            keep = ("value", "unit", "ms_per_step", "step_ms_median", "step_ms_min", "warm_step_ms_median",
                    "plan_ms", "plan_lifecycle_ms", "one_shot_ms", "launch_floor_us", "hbm_gbps", "hbm_frac",
                    "hbm_frac_median_step", "mfma_util", "mfma_util_cap", "config", "roofline", "ablation",
                    "parity")
            out["also"] = []
            for n in (int(v) for v in args.also.split(",")):
                o = measure(args, n, True)
                e = {k: o[k] for k in keep if k in o}
                # the nested summaries stay short: the full objects come from `--workload n`
                e["config"] = {k: o["config"][k] for k in ("workload", "H", "storage", "tokens_per_step", "slots")}
                e["roofline"] = {k: o["roofline"][k] for k in ("kernel", "achieved", "frac", "traffic", "traffic_source",
                                                              "algorithmic_bytes_per_launch", "avg_launch_us",
                                                              "other_kernel", "slots_per_launch")}
                e["parity"] = {k: o["parity"][k] for k in ("slots_checked", "tokens_checked_per_slot", "rel_l2", "max_abs")}
                out["also"].append(e)
    except RuntimeError as e:
        print(f"bench.py: {e}", file=sys.stderr)
        return 1
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
