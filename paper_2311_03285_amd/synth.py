"""Seeded synthetic inputs for heterogeneous batched LoRA over a paged pool.

This module only *draws inputs*: page placements, adapter ranks, weight bit patterns,
activations, token->adapter ids and request segments.  It contains none of the LoRA
arithmetic (no decode of 16-bit patterns to numbers, no dot products); both the GPU
library's tests/bench and the CPU oracle's tests are fed from here so that the two sides
consume identical bits.

Shapes follow the paper's evaluation set-up: hidden sizes and rank sets of its model
table (Table 1), adapter counts and length ranges of its workload table (Table 2), the
power-law adapter popularity of Sec. 7.1, LoRA on the q/k/v/o projections (Sec. 2), and
the unified pool where a page is one H-vector and a rank-r matrix occupies r pages that
are interleaved with KV-cache pages (Sec. 5.1, Fig. 3).

Every value is a pure function of (seed, coordinates): weights of (adapter, slot, A|B)
can be regenerated without materialising the pool on the host.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

F16 = 0
BF16 = 1

_SEED_BASE = 20231103 * 10

# stream tags (second Philox key word, high bits)
_TAG_PLACEMENT = 1
_TAG_RANKS = 2
_TAG_IDS = 3
_TAG_LENGTHS = 4
_TAG_WEIGHT = 5
_TAG_X = 6
_TAG_Y = 7
_TAG_POPULARITY = 8
_TAG_MISC = 9


def _rng(seed: int, tag: int, a: int = 0, b: int = 0, c: int = 0) -> np.random.Generator:
    """Counter-based generator keyed by (seed, tag, a, b, c)."""
    k0 = (int(seed) & 0xFFFFFFFFFFFFFFFF)
    tag, a, b, c = int(tag), int(a), int(b), int(c)
    k1 = ((tag & 0xFF) << 56) | ((a & 0xFFFFFF) << 32) | ((b & 0xFFFF) << 16) | (c & 0xFFFF)
    return np.random.Generator(np.random.Philox(key=np.array([k0, k1], dtype=np.uint64)))


def round_to_bits(values: np.ndarray, dtype: int) -> np.ndarray:
    """Round real values to the 16-bit storage type (nearest-even) and return the raw bits."""
    if dtype == F16:
        return np.ascontiguousarray(values, dtype=np.float32).astype(np.float16).view(np.uint16)
    if dtype == BF16:
        f = np.ascontiguousarray(values, dtype=np.float32).view(np.uint32)
        # nearest-even on the 16 discarded bits (inputs are finite)
        bias = np.uint32(0x7FFF) + ((f >> np.uint32(16)) & np.uint32(1))
        return ((f + bias) >> np.uint32(16)).astype(np.uint16)
    raise ValueError("dtype must be F16 or BF16")


def nan_bits(dtype: int) -> int:
    """A quiet-NaN bit pattern of the storage type (canary for pages no adapter owns)."""
    return 0x7E00 if dtype == F16 else 0x7FC0


def popularity(n_adapters: int, alpha: float, seed: int, law: str = "power") -> np.ndarray:
    """Probability of each adapter being requested (Sec. 7.1: power law with exponent alpha).

    law="power": weights w = u**(1/alpha), u ~ U(0,1] i.i.d. (density alpha*w**(alpha-1));
                 smaller alpha concentrates requests on few adapters, as the paper's
                 ablation on alpha describes.
    law="zipf" : p_i proportional to (i+1)**(-alpha), a more skewed stress case.
    """
    if law == "power":
        u = 1.0 - _rng(seed, _TAG_POPULARITY).random(n_adapters)
        w = u ** (1.0 / alpha)
    elif law == "zipf":
        w = (np.arange(n_adapters, dtype=np.float64) + 1.0) ** (-alpha)
    elif law == "uniform":
        w = np.ones(n_adapters)
    else:
        raise ValueError(law)
    return w / w.sum()


@dataclass
class Workload:
    """One synthetic batch plus the adapters resident in the pool.

    page_idx[a] has shape (n_slots, 2, rank[a]): [slot][0] are the pages holding the r
    columns of A, [slot][1] the pages holding the r rows of B.
    seg_offsets is None for a pure decode batch (every token its own segment).
    """
    name: str
    seed: int
    H: int
    dtype: int
    n_pages: int
    n_slots: int
    ranks: np.ndarray                      # int32 [n_adapters]
    page_idx: List[np.ndarray]             # per adapter int32 [n_slots, 2, r]
    ids: np.ndarray                        # int32 [T], -1 = no adapter
    seg_offsets: Optional[np.ndarray]      # int32 [n_seg+1] or None
    batch_seed: int = 0                    # keys ids / lengths / x / y (seed keys the pool)
    y_zero: bool = False                   # y_in = 0 instead of N(0,1)
    int_valued: bool = False               # small-integer x / weights (exact in fp32)
    _cache: Dict[Tuple[int, int, int], np.ndarray] = field(default_factory=dict, repr=False)

    @property
    def T(self) -> int:
        return int(self.ids.shape[0])

    @property
    def n_adapters(self) -> int:
        return int(self.ranks.shape[0])

    def used_adapters(self) -> np.ndarray:
        u = np.unique(self.ids)
        return u[u >= 0].astype(np.int32)

    # ---- values -------------------------------------------------------------------
    def weight_bits(self, adapter: int, slot: int, which: int) -> np.ndarray:
        """uint16 [r, H]: row j is page j of A (which=0: column j of A) or B (which=1: row j)."""
        r = int(self.ranks[adapter])
        g = _rng(self.seed, _TAG_WEIGHT, adapter, slot, which)
        if r == 0:
            return np.zeros((0, self.H), dtype=np.uint16)
        if self.int_valued:
            v = g.integers(-2, 3, size=(r, self.H)).astype(np.float32)
        else:
            v = g.standard_normal((r, self.H), dtype=np.float32)
            # A ~ N(0, 1/H), B ~ N(0, 1/r)  (variances)
            v *= np.float32(1.0 / np.sqrt(self.H if which == 0 else r))
        return round_to_bits(v, self.dtype)

    def x_bits(self, slot: int = 0) -> np.ndarray:
        g = _rng(self.batch_seed, _TAG_X, slot)
        if self.int_valued:
            v = g.integers(-2, 3, size=(self.T, self.H)).astype(np.float32)
        else:
            v = g.standard_normal((self.T, self.H), dtype=np.float32)
        return round_to_bits(v, self.dtype)

    def y_in(self, slot: int = 0) -> np.ndarray:
        if self.y_zero:
            return np.zeros((self.T, self.H), dtype=np.float32)
        g = _rng(self.batch_seed, _TAG_Y, slot)
        if self.int_valued:
            return g.integers(-4, 5, size=(self.T, self.H)).astype(np.float32)
        return g.standard_normal((self.T, self.H), dtype=np.float32)

    def y16_bits(self, slot: int = 0) -> np.ndarray:
        """The same y_in as an input of the storage type (for the 16-bit-output variant)."""
        return round_to_bits(self.y_in(slot), self.dtype)

    # ---- host views of the pool ------------------------------------------------------
    def adapter_page_list(self, adapter: int) -> np.ndarray:
        """Flat int32 list ordered [slot][A pages j=0..r-1][B pages j=0..r-1]."""
        return np.ascontiguousarray(self.page_idx[adapter], dtype=np.int32).reshape(-1)

    def owned_pages(self) -> np.ndarray:
        if not self.page_idx:
            return np.zeros(0, dtype=np.int32)
        return np.concatenate([p.reshape(-1) for p in self.page_idx]).astype(np.int32)

    def dense_pool_bits(self, adapters: Optional[Sequence[int]] = None) -> np.ndarray:
        """uint16 [n_pages, H] host image: NaN canaries everywhere, weights on owned pages.

        Only for pools small enough for host memory.
        """
        pool = np.full((self.n_pages, self.H), nan_bits(self.dtype), dtype=np.uint16)
        todo = range(self.n_adapters) if adapters is None else adapters
        for a in todo:
            for s in range(self.n_slots):
                for w in (0, 1):
                    pool[self.page_idx[a][s, w]] = self.weight_bits(a, s, w)
        return pool

    def compact_pool(self, slot: int, adapters: Optional[Sequence[int]] = None):
        """Pages of one slot of the given adapters packed into a small host pool.

        Returns (rows uint16 [n_rows, H], lists) where lists[a] = int32 [2, r] row numbers
        inside `rows` for adapter a (A pages, B pages).  A re-paging of the same weights,
        used when the real pool does not fit in host memory.
        """
        todo = list(self.used_adapters() if adapters is None else adapters)
        n_rows = int(sum(2 * int(self.ranks[a]) for a in todo))
        rows = np.empty((n_rows, self.H), dtype=np.uint16)
        lists: Dict[int, np.ndarray] = {}
        at = 0
        for a in todo:
            r = int(self.ranks[a])
            l = np.arange(at, at + 2 * r, dtype=np.int32).reshape(2, r)
            rows[l[0]] = self.weight_bits(a, slot, 0)
            rows[l[1]] = self.weight_bits(a, slot, 1)
            lists[int(a)] = l
            at += 2 * r
        return rows, lists

    # ---- accounting -------------------------------------------------------------------
    def algorithmic_bytes(self) -> int:
        """Minimum HBM bytes for one slot: each distinct adapter's A and B pages once,
        x once, y read + written once (fp32)."""
        eb = 2
        used = self.used_adapters()
        pages = int(sum(2 * int(self.ranks[a]) for a in used)) * self.H * eb
        t_act = int(np.count_nonzero(self.ids >= 0))
        return pages + t_act * self.H * eb + 2 * t_act * self.H * 4

    def shrink_bytes(self) -> int:
        used = self.used_adapters()
        t_act = int(np.count_nonzero(self.ids >= 0))
        return int(sum(int(self.ranks[a]) for a in used)) * self.H * 2 + t_act * self.H * 2

    def expand_bytes(self) -> int:
        used = self.used_adapters()
        t_act = int(np.count_nonzero(self.ids >= 0))
        return int(sum(int(self.ranks[a]) for a in used)) * self.H * 2 + 2 * t_act * self.H * 4

    def flops(self) -> int:
        """2rH (shrink) + 2rH (expand) per token, one slot."""
        r_tok = self.ranks[self.ids[self.ids >= 0]].astype(np.int64)
        return int(4 * self.H * r_tok.sum())


def _place(seed: int, n_pages: int, ranks: np.ndarray, n_slots: int) -> List[np.ndarray]:
    """Distinct random page indices for every (adapter, slot, A|B, j)."""
    total = int(2 * n_slots * ranks.astype(np.int64).sum())
    if total > n_pages:
        raise ValueError(f"pool of {n_pages} pages cannot hold {total} adapter pages")
    g = _rng(seed, _TAG_PLACEMENT)
    if total * 4 >= n_pages:
        picks = g.permutation(n_pages)[:total]
    else:
        picks = g.choice(n_pages, size=total, replace=False, shuffle=True)
    picks = picks.astype(np.int32)
    out, at = [], 0
    for r in ranks:
        n = 2 * n_slots * int(r)
        out.append(picks[at:at + n].reshape(n_slots, 2, int(r)).copy())
        at += n
    return out


def make_workload(name: str, seed: int, H: int, dtype: int, n_pages: int, n_slots: int,
                  ranks: Sequence[int], ids: Sequence[int],
                  seg_offsets: Optional[Sequence[int]] = None, *, batch_seed: Optional[int] = None,
                  y_zero: bool = False, int_valued: bool = False) -> Workload:
    ranks = np.asarray(ranks, dtype=np.int32)
    return Workload(name=name, seed=seed, H=H, dtype=dtype, n_pages=n_pages, n_slots=n_slots,
                    ranks=ranks, page_idx=_place(seed, n_pages, ranks, n_slots),
                    ids=np.asarray(ids, dtype=np.int32),
                    seg_offsets=None if seg_offsets is None else np.asarray(seg_offsets, dtype=np.int32),
                    batch_seed=seed if batch_seed is None else batch_seed,
                    y_zero=y_zero, int_valued=int_valued)


def _segments(seed: int, n_req: int, lo: int, hi: int) -> np.ndarray:
    g = _rng(seed, _TAG_LENGTHS)
    lens = g.integers(lo, hi + 1, size=n_req)
    return np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)


def _ids_for_segments(seg_offsets: np.ndarray, seg_adapter: np.ndarray) -> np.ndarray:
    return np.repeat(seg_adapter.astype(np.int32), np.diff(seg_offsets)).astype(np.int32)


def config(n: int, *, batch: int = 0, law: str = "power", **kw) -> Workload:
    """The five benchmark configurations.  `batch` re-draws the batch (ids, lengths, x, y)
    against the same resident adapters, for rotating over distinct batches when timing."""
    seed = _SEED_BASE + n
    bseed = seed + 1000 * batch          # batch-level draws
    kw["batch_seed"] = bseed
    if n == 1:
        ranks = np.array([4, 4, 8, 8], dtype=np.int32)
        ids = _rng(bseed, _TAG_IDS).integers(0, 4, size=8)
        w = make_workload("cfg1-tiny-decode", seed, 256, F16, 64, 1, ranks, ids, **kw)
    elif n == 2:
        ranks = _rng(seed, _TAG_RANKS).choice([8, 16, 32, 64], size=32)
        ids = _rng(bseed, _TAG_IDS).integers(0, 32, size=32)
        w = make_workload("cfg2-llama7b-decode", seed, 4096, F16, 65536, 1, ranks, ids, **kw)
    elif n == 3:
        ranks = _rng(seed, _TAG_RANKS).choice([8, 16, 32, 64, 128], size=200)
        seg = _segments(bseed, 16, 64, 512)
        p = popularity(200, 1.0, seed, law)
        seg_ad = _rng(bseed, _TAG_IDS).choice(200, size=16, p=p)
        w = make_workload("cfg3-prefill", seed, 4096, F16, 1 << 18, 4, ranks,
                          _ids_for_segments(seg, seg_ad), seg, **kw)
    elif n == 4:
        ranks = _rng(seed, _TAG_RANKS).choice([8, 16, 32, 64], size=2000)
        p = popularity(2000, 1.0, seed, law)
        ids = _rng(bseed, _TAG_IDS).choice(2000, size=256, p=p)
        n_pages = int(0.4 * 288e9) // (5120 * 2)
        w = make_workload("cfg4-large-pool-decode", seed, 5120, F16, n_pages, 4, ranks, ids, **kw)
    elif n == 5:
        ranks = _rng(seed, _TAG_RANKS).choice([16, 32, 64, 128], size=1000)
        seg_p = _segments(bseed, 8, 128, 1024)
        n_dec = 192
        seg = np.concatenate([seg_p, seg_p[-1] + 1 + np.arange(n_dec)]).astype(np.int32)
        seg_ad = _rng(bseed, _TAG_IDS).integers(0, 1000, size=8 + n_dec)
        w = make_workload("cfg5-mixed", seed, 8192, BF16, 1 << 22, 16, ranks,
                          _ids_for_segments(seg, seg_ad), seg, **kw)
    else:
        raise ValueError("config number must be 1..5")
    return w
