"""The seeded input generators: determinism, shapes, structure (no LoRA arithmetic here)."""
import numpy as np
import pytest

from paper_2311_03285_amd import synth


def test_round_to_bits_f16_matches_numpy():
    v = np.random.default_rng(0).standard_normal(1000)
    assert np.array_equal(synth.round_to_bits(v, synth.F16), v.astype(np.float32).astype(np.float16).view(np.uint16))


def test_round_to_bits_bf16_nearest_even():
    one = np.float32(1.0).view(np.uint32)
    cases = {
        one + 0x7FFF: 0x3F80,          # below half: down
        one + 0x8000: 0x3F80,          # tie, even stays
        one + 0x8001: 0x3F81,          # above half: up
        one + 0x18000: 0x3F82,         # tie, odd rounds up to even
    }
    for f, b in cases.items():
        val = np.array([f], dtype=np.uint32).view(np.float32)
        assert synth.round_to_bits(val, synth.BF16)[0] == b


@pytest.mark.parametrize("n", [1, 2, 3, 4, 5])
def test_configs_are_deterministic_and_well_formed(n):
    a, b = synth.config(n), synth.config(n)
    assert np.array_equal(a.ids, b.ids) and np.array_equal(a.ranks, b.ranks)
    pages = a.owned_pages()
    assert pages.size == 2 * a.n_slots * int(a.ranks.sum())
    assert np.unique(pages).size == pages.size, "page indices must be distinct"
    assert pages.min() >= 0 and pages.max() < a.n_pages
    assert a.ids.min() >= 0 and a.ids.max() < a.n_adapters
    if a.seg_offsets is not None:
        s = a.seg_offsets
        assert s[0] == 0 and s[-1] == a.T and np.all(np.diff(s) > 0)
        for i in range(len(s) - 1):
            assert np.all(a.ids[s[i]:s[i + 1]] == a.ids[s[i]])
    u = int(a.used_adapters()[0])
    assert np.array_equal(a.weight_bits(u, 0, 1), b.weight_bits(u, 0, 1))
    assert a.weight_bits(u, 0, 0).shape == (a.ranks[u], a.H)


def test_config_sizes_follow_the_stated_shapes():
    c1 = synth.config(1)
    assert (c1.H, c1.n_pages, c1.T, list(c1.ranks)) == (256, 64, 8, [4, 4, 8, 8])
    c2 = synth.config(2)
    assert (c2.H, c2.n_pages, c2.T, c2.n_adapters) == (4096, 65536, 32, 32)
    assert set(c2.ranks) <= {8, 16, 32, 64}
    c3 = synth.config(3)
    lens = np.diff(c3.seg_offsets)
    assert len(lens) == 16 and lens.min() >= 64 and lens.max() <= 512 and c3.n_slots == 4
    c4 = synth.config(4)
    assert c4.H == 5120 and c4.T == 256 and c4.n_adapters == 2000 and c4.n_slots == 4
    assert abs(c4.n_pages * 5120 * 2 - 0.4 * 288e9) < 5120 * 2
    c5 = synth.config(5)
    lens = np.diff(c5.seg_offsets)
    assert c5.dtype == synth.BF16 and c5.n_slots == 16 and (lens == 1).sum() == 192
    assert lens[:8].min() >= 128 and lens[:8].max() <= 1024


def test_rotating_batches_keep_the_pool_and_redraw_the_batch():
    a, b = synth.config(4, batch=0), synth.config(4, batch=3)
    assert np.array_equal(a.ranks, b.ranks)
    assert all(np.array_equal(p, q) for p, q in zip(a.page_idx[:50], b.page_idx[:50]))
    assert not np.array_equal(a.ids, b.ids)
    assert np.array_equal(a.weight_bits(7, 2, 1), b.weight_bits(7, 2, 1))
    assert not np.array_equal(a.x_bits()[:2], b.x_bits()[:2])


def test_popularity_laws():
    p = synth.popularity(2000, 1.0, 1)
    z = synth.popularity(2000, 1.0, 1, "zipf")
    assert abs(p.sum() - 1) < 1e-12 and abs(z.sum() - 1) < 1e-12
    # smaller alpha => more concentrated (the paper's ablation on alpha)
    top = lambda q: np.sort(q)[::-1][:20].sum()
    assert top(synth.popularity(2000, 0.1, 1)) > top(synth.popularity(2000, 1.0, 1))
    assert z[0] > z[1] > z[100]
