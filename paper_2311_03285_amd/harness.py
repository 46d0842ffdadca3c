"""Test / bench plumbing: puts a synthetic workload on the GPU through the C ABI.

PyTorch is used only to own device memory and streams.  Nothing here computes any part of
the LoRA path; weights go in through slora_pool_write_pages and every result comes out of
the library's kernels.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from typing import Dict, Iterable, List, Optional, Sequence

import numpy as np
import torch

from . import slora, synth


def _torch_dtype(dtype: int):
    return torch.float16 if dtype == synth.F16 else torch.bfloat16


def bits_to_device(bits: np.ndarray, device) -> torch.Tensor:
    """uint16 patterns -> int16 device tensor with the same bits."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(device)


class DeviceWorkload:
    """A synth.Workload resident on the GPU: pool tensor, library pool handle, adapters loaded.

    real_adapters: adapters whose pages get their seeded, oracle-visible weights (default: the
    adapters the batch uses; pass "all" for every adapter).  Pages of other adapters are
    filled on the device with arbitrary finite values; all remaining pages are marked as KV
    cache and hold NaN.
    """

    def __init__(self, w: synth.Workload, device="cuda:0", real_adapters="used", slots: Optional[Sequence[int]] = None,
                 max_rank: Optional[int] = None, mark_kv: bool = True, threads: int = 8):
        self.w = w
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.real_slots = list(range(w.n_slots)) if slots is None else list(slots)
        self.pool_t = torch.empty((w.n_pages, w.H), dtype=torch.int16, device=self.device)
        nanv = synth.nan_bits(w.dtype)
        self.pool_t.fill_(nanv - 65536 if nanv >= 32768 else nanv)
        self.pool = slora.pool_init(w.H, w.n_pages, w.dtype, self.pool_t.data_ptr(), w.n_slots,
                                    int(max(int(w.ranks.max()) if w.n_adapters else 0, 1) if max_rank is None else max_rank))
        self.plans: List = []
        if isinstance(real_adapters, str):
            real = set(range(w.n_adapters)) if real_adapters == "all" else set(int(a) for a in w.used_adapters())
        else:
            real = set(int(a) for a in real_adapters)
        self.real = real
        for a in range(w.n_adapters):
            slora.adapter_load(self.pool, a, int(w.ranks[a]), w.adapter_page_list(a))
        if mark_kv:
            owned = w.owned_pages()
            free = np.ones(w.n_pages, dtype=bool)
            free[owned] = False
            slora.pool_mark_kv(self.pool, np.nonzero(free)[0].astype(np.int32), True)
        self._fill_filler([a for a in range(w.n_adapters) if a not in real])
        self._write_real(sorted(real), threads)
        torch.cuda.synchronize(self.device)

    # -- pages of adapters the batch does not use: finite filler generated on the device
    def _fill_filler(self, adapters: List[int], chunk_pages: int = 1 << 15) -> None:
        if not adapters:
            return
        w = self.w
        pages = np.concatenate([w.page_idx[a].reshape(-1) for a in adapters]).astype(np.int32)
        g = torch.Generator(device=self.device)
        g.manual_seed(w.seed & 0x7FFFFFFF)
        for at in range(0, pages.size, chunk_pages):
            idx = pages[at:at + chunk_pages]
            src = (torch.randn((idx.size, w.H), device=self.device, generator=g) * 0.05).to(_torch_dtype(w.dtype))
            slora.pool_write_pages(self.pool, idx, src.data_ptr(), True)
            del src

    def _write_real(self, adapters: List[int], threads: int, chunk_adapters: int = 64) -> None:
        w = self.w

        def gen(a):
            out = []
            for s in self.real_slots:
                out.append((w.page_idx[a][s, 0], w.weight_bits(a, s, 0)))
                out.append((w.page_idx[a][s, 1], w.weight_bits(a, s, 1)))
            return out

        with ThreadPoolExecutor(max_workers=threads) as ex:
            for at in range(0, len(adapters), chunk_adapters):
                parts = [p for res in ex.map(gen, adapters[at:at + chunk_adapters]) for p in res]
                parts = [p for p in parts if p[0].size]
                if not parts:
                    continue
                idx = np.concatenate([p[0] for p in parts]).astype(np.int32)
                bits = np.concatenate([p[1] for p in parts])
                slora.pool_write_pages(self.pool, idx, bits, False)

    # -- batch tensors -----------------------------------------------------------------
    def x_dev(self, slot: int = 0) -> torch.Tensor:
        return bits_to_device(self.w.x_bits(slot), self.device)

    def y_dev(self, slot: int = 0) -> torch.Tensor:
        return torch.from_numpy(self.w.y_in(slot)).to(self.device)

    def plan(self, ids=None, seg_offsets="workload"):
        ids = self.w.ids if ids is None else ids
        seg = self.w.seg_offsets if isinstance(seg_offsets, str) else seg_offsets
        p = slora.batch_plan(self.pool, ids, seg)
        self.plans.append(p)
        return p

    def gather(self, adapter: int, slot: int, which: int) -> np.ndarray:
        r = int(self.w.ranks[adapter])
        out = torch.empty((max(r, 1), self.w.H), dtype=torch.int16, device=self.device)
        slora.adapter_gather(self.pool, adapter, slot, which, out.data_ptr())
        torch.cuda.synchronize(self.device)
        return out[:r].cpu().numpy().view(np.uint16)

    def close(self) -> None:
        torch.cuda.synchronize(self.device)
        for p in self.plans:
            slora.plan_destroy(p)
        self.plans = []
        if self.pool is not None:
            slora.pool_destroy(self.pool)
            self.pool = None
        self.pool_t = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()
