// Batch scheduler: turns (adapter id per token, request segments) into device work lists.
//
// The paper batches requests of different adapters and ranks in one iteration (Sec. 4.1) and
// runs the LoRA term with kernels that take no padding (Sec. 5.3); how the work is ordered is
// left open there.  Here tokens are grouped by adapter so that each adapter's pages are
// streamed once per group, groups are ordered by rank (longest work first, so the tail of a
// launch is made of short items), and each group goes either to the wavefront-reduction
// matrix-vector kernels (few tokens: decode) or to the MFMA kernels (many tokens: prefill).
// A plan depends only on the ids, so one plan serves every projection of every layer.
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cstdint>
#include <cstring>
#include <new>

#include "slora_internal.hpp"

using namespace slora;

namespace {

struct Group {
    int32_t id;
    int32_t rank;
    int64_t arena_off;
    int32_t first_tok;
    std::vector<int32_t> toks;
};

int32_t hip_fail(hipError_t e, const char *what) { return fail(SLORA_EHIP, "%s: %s", what, hipGetErrorString(e)); }

// Lay an MFMA work list out for the 8 XCDs.  The list arrives in group order (all items of an
// adapter adjacent, adapters by descending rank).  It is cut into kXcds runs of about equal
// cost (bytes moved), run k becomes column k of a row-major table with kXcds columns, short
// columns are padded with empty items (ntok == 0).  The kernels map workgroup ids so that
// column k runs on XCD k: the tiles of one adapter share an L2 and its pages are fetched
// from HBM once per XCD instead of once per tile.  A big adapter may straddle two columns.
template <class Cost>
void xcd_layout(std::vector<Item> &items, Cost cost, bool group)
{
    if (items.empty()) return;
    if (!group) { // plain order: consecutive items go to consecutive XCDs; pad the last row
        items.resize((items.size() + kXcds - 1) / kXcds * kXcds, Item{0, 0, 0, 0, 0, 0, 0, 0});
        return;
    }
    int64_t total = 0;
    for (const Item &i : items) total += cost(i);
    std::vector<std::vector<Item>> col((size_t)kXcds);
    int64_t seen = 0;
    for (const Item &i : items) {
        // column of the item's midpoint in the running cost
        const int64_t c = cost(i);
        int k = (int)(((seen + c / 2) * kXcds) / std::max<int64_t>(total, 1));
        k = std::min(std::max(k, 0), kXcds - 1);
        col[(size_t)k].push_back(i);
        seen += c;
    }
    size_t rows = 0;
    for (const auto &c : col) rows = std::max(rows, c.size());
    std::vector<Item> out(rows * (size_t)kXcds, Item{0, 0, 0, 0, 0, 0, 0, 0});
    for (int k = 0; k < kXcds; ++k)
        for (size_t r = 0; r < col[(size_t)k].size(); ++r) out[r * (size_t)kXcds + (size_t)k] = col[(size_t)k][r];
    items.swap(out);
}

} // namespace

int32_t slora::build_plan(slora_pool *pool, slora_plan *plan, const int32_t *ids, int32_t T,
                          const int32_t *seg_offsets, int32_t n_seg)
{
    // ---- validate ----------------------------------------------------------------------
    if (T < 0) return fail(SLORA_EINVAL, "T=%d must be >= 0", T);
    if (T > 0 && !ids) return fail(SLORA_EINVAL, "token_adapter_ids is NULL");
    if (seg_offsets) {
        if (n_seg < 0) return fail(SLORA_ESEG, "n_seg=%d must be >= 0", n_seg);
        if (seg_offsets[0] != 0) return fail(SLORA_ESEG, "seg_offsets[0]=%d must be 0", seg_offsets[0]);
        if (seg_offsets[n_seg] != T)
            return fail(SLORA_ESEG, "seg_offsets[n_seg]=%d must equal T=%d", seg_offsets[n_seg], T);
        for (int32_t s = 0; s < n_seg; ++s) {
            if (seg_offsets[s + 1] <= seg_offsets[s] || seg_offsets[s + 1] > T)
                return fail(SLORA_ESEG, "seg_offsets must be strictly increasing and end at T (segment %d)", s);
            const int32_t id0 = ids[seg_offsets[s]];
            for (int32_t t = seg_offsets[s] + 1; t < seg_offsets[s + 1]; ++t)
                if (ids[t] != id0)
                    return fail(SLORA_ESEG, "token %d has id %d but its segment %d starts with id %d", t, ids[t], s, id0);
        }
    }
    std::unordered_map<int32_t, int32_t> group_of;
    std::vector<Group> groups;
    try {
        for (int32_t t = 0; t < T; ++t) {
            const int32_t id = ids[t];
            if (id == -1) continue;
            auto g = group_of.find(id);
            if (g == group_of.end()) {
                auto a = pool->adapters.find(id);
                if (id < 0 || a == pool->adapters.end())
                    return fail(SLORA_ENOENT, "token %d names adapter %d, which is not loaded", t, id);
                group_of.emplace(id, (int32_t)groups.size());
                groups.push_back(Group{id, a->second.rank, a->second.arena_off, t, {}});
                g = group_of.find(id);
            }
            groups[(size_t)g->second].toks.push_back(t);
        }

        // ---- order: rank bucket (descending), then more tokens first, then first appearance --
        std::vector<int32_t> order;
        for (int32_t g = 0; g < (int32_t)groups.size(); ++g)
            if (groups[(size_t)g].rank > 0) order.push_back(g);
        std::sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
            const Group &x = groups[(size_t)a], &y = groups[(size_t)b];
            if (x.rank != y.rank) return x.rank > y.rank;
            if (x.toks.size() != y.toks.size()) return x.toks.size() > y.toks.size();
            return x.first_tok < y.first_tok;
        });

        plan->T = T;
        plan->tok_idx.clear();
        plan->vs_items.clear();
        plan->ve_items.clear();
        plan->ms_items.clear();
        plan->mj_items.clear();
        plan->me_items.clear();
        plan->sum_rank = 0;
        plan->n_groups = (int32_t)order.size();
        plan->n_groups_vec = plan->n_groups_mfma = 0;
        plan->n_mfma_tiles = 0;
        plan->n_sync = 0;
        plan->ms_max_nj = 0;
        plan->part_floats = 0;
        plan->max_shrink_tok = 0;
        const int32_t n_chunks = (pool->H + kMsGranule - 1) / kMsGranule;
        int32_t max_rank = 0;
        const int32_t H = pool->H;
        // The MFMA kernels pay off when adapters have many tokens AND there are enough 32-token
        // tiles to fill the GPU: a handful of tiles is a few long, latency-bound workgroups, and
        // such groups are faster on the vector path (their pages are re-read from L2).
        int64_t mfma_tiles = 0;
        for (int32_t gi : order) {
            const int64_t n = (int64_t)groups[(size_t)gi].toks.size();
            if (n >= pool->mfma_min_tokens) mfma_tiles += (n + kMfmaTok - 1) / kMfmaTok;
        }
        const int64_t min_tokens = mfma_tiles >= pool->mfma_min_tiles ? pool->mfma_min_tokens : INT64_MAX;
        // Size of a share of an MFMA shrink tile (see below): mfma_split_bytes, or more when the
        // batch is so large that shares of that size would be far more than the GPU can hold at a
        // time (every share of a split tile costs a set of partial sums) - about three workgroups
        // per compute unit for a launch of up to eight slots.
        int64_t ms_bytes = 0;
        for (int32_t gi : order) {
            const Group &g = groups[(size_t)gi];
            const int64_t n = (int64_t)g.toks.size();
            if (n < min_tokens) continue;
            const int64_t n_tok_tiles = (n + kMsTok - 1) / kMsTok, n_rank_blocks = (g.rank + kMsRanks - 1) / kMsRanks;
            ms_bytes += (n * n_rank_blocks + (int64_t)g.rank * n_tok_tiles) * H * 2;
        }
        const int64_t launch_slots = std::min<int64_t>(pool->n_slots, SLORA_MAX_MULTI);
        const int64_t share_bytes = std::max<int64_t>(pool->mfma_split_bytes, ms_bytes * launch_slots / (3 * 256));
        int32_t n_vec_groups = 0;
        for (int32_t gi : order)
            if ((int64_t)groups[(size_t)gi].toks.size() < min_tokens) n_vec_groups++;
        // vector-expand items: long runs of columns, halved while a launch would have fewer
        // workgroups than the GPU has CUs
        int32_t chunks = (H + kExpandColsMax - 1) / kExpandColsMax;
        auto cols_of = [&](int32_t c) { return ((H + c - 1) / c + 511) / 512 * 512; };
        while ((int64_t)n_vec_groups * chunks < 256 && cols_of(chunks) > 512) chunks *= 2;
        int32_t ecols = cols_of(chunks);
        // still short of workgroups at the smallest items: split the ranks over the wavefronts
        plan->expand_split = ecols == 512 && (int64_t)n_vec_groups * chunks < 512;
        // the vector shrink stages its tokens' x rows in LDS: at most 64 KiB of them per item
        const int32_t shrink_tok = std::max(1, std::min(kShrinkTok, 65536 / (H * 2)));
        const int32_t shrink_pages = (int32_t)pool->shrink_pages;
        plan->expand_threads = ecols / 8;
        // One launch for both stages of decode groups (at most kExpandTok tokens): a workgroup per
        // group streams the whole adapter.  That pays when the batch has enough groups to fill
        // the GPU about three times over with whole-group workgroups AND the groups are large
        // (a workgroup's waits for its work item, page lists and first pages are then short beside
        // its streaming): measured per step inside one process, 2.41 -> 2.38 ms on the mixed
        // configuration (H = 8192, 2.3 MB of pages per group); on the large-pool decode one (0.6 MB
        // per group) 109.0 -> 112.3 us in one process and 111.7 -> 110.8 us in the next.
        // x rows are staged in LDS (64 KiB: H <= 8192).
        int64_t n_small = 0, small_bytes = 0;
        for (int32_t gi : order) {
            const int64_t n = (int64_t)groups[(size_t)gi].toks.size();
            if (n < min_tokens && n <= kExpandTok) {
                n_small++;
                small_bytes += (int64_t)groups[(size_t)gi].rank * H * 4; // A and B pages
            }
        }
        const bool fuse = pool->fuse_decode != 0 && H <= 8192 &&
                          (pool->fuse_decode > 1 ||
                           (n_small * launch_slots >= 3 * 256 && small_bytes >= n_small * (int64_t(1) << 20)));
        std::vector<Item> vs_tail, ve_tail;
        plan->vf_items.clear();
        for (int32_t gi : order) {
            const Group &g = groups[(size_t)gi];
            const int32_t n = (int32_t)g.toks.size();
            const int32_t pos_base = (int32_t)plan->tok_idx.size();
            plan->tok_idx.insert(plan->tok_idx.end(), g.toks.begin(), g.toks.end());
            plan->sum_rank += g.rank;
            max_rank = std::max(max_rank, g.rank);
            const int32_t off = (int32_t)g.arena_off;
            if ((int64_t)n >= min_tokens) {
                plan->n_groups_mfma++;
                // v tiles of 32 tokens, numbered in order; an expand item covers one tile, a shrink
                // item up to four consecutive ones (its pages are then read once for them all)
                const int32_t tile0 = plan->n_mfma_tiles;
                const int32_t n_tiles = (n + kMfmaTok - 1) / kMfmaTok;
                plan->n_mfma_tiles += n_tiles;
                for (int32_t p = 0; p < n; p += kMsTok) {
                    const int32_t nt = std::min(kMsTok, n - p);
                    for (int32_t j = 0; j < g.rank; j += kMsRanks) {
                        const int32_t nj = std::min(kMsRanks, g.rank - j);
                        // Shares of H: a workgroup streams its rows at a rate set by what it keeps in
                        // flight, so a tile of (nt + nj) rows x H is cut into shares of about
                        // share_bytes each - the launch then consists of many workgroups of
                        // similar, small size and every compute unit is busy to the end.  A share is
                        // never shorter than mfma_split_min_h elements: the partial sums a share
                        // leaves behind (and the last one reads back) must stay small beside its rows.
                        const int64_t cost = (int64_t)(nt + nj) * H * 2;
                        int64_t parts = (cost + share_bytes / 2) / share_bytes;
                        parts = std::min<int64_t>(parts, H / std::max<int64_t>(pool->mfma_split_min_h, kMsGranule));
                        parts = std::min<int64_t>(parts, std::min<int64_t>(n_chunks, 64));
                        const int64_t mb = (nt + 31) / 32, nb = (nj + 31) / 32;
                        if (parts < 2 || plan->part_floats + parts * mb * nb * 1024 > (int64_t(1) << 30))
                            parts = 1;
                        plan->ms_max_nj = std::max(plan->ms_max_nj, nj);
                        MsItem it{};
                        it.arena_off = off;
                        it.rank = g.rank;
                        it.j0 = j;
                        it.nj = nj;
                        it.pos0 = pos_base + p;
                        it.ntok = nt;
                        it.tile = tile0 + p / kMfmaTok;
                        it.n_parts = (int32_t)parts;
                        it.sync = -1;
                        if (parts > 1) {
                            it.sync = plan->n_sync++;
                            it.part_off = (int32_t)plan->part_floats;
                            plan->part_floats += parts * mb * nb * 1024;
                            plan->mj_items.push_back(it);
                        }
                        for (int32_t q = 0; q < (int32_t)parts; ++q) {
                            it.part = q;
                            it.c0 = (int32_t)((int64_t)n_chunks * q / parts);
                            it.c1 = (int32_t)((int64_t)n_chunks * (q + 1) / parts);
                            plan->ms_items.push_back(it);
                        }
                    }
                }
                for (int32_t t = 0; t < n_tiles; ++t) {
                    const int32_t p = t * kMfmaTok;
                    const int32_t nt = std::min(kMfmaTok, n - p);
                    for (int32_t c = 0; c < H; c += kMfmaExpandCols)
                        plan->me_items.push_back(
                            Item{off, g.rank, c, std::min(kMfmaExpandCols, H - c), pos_base + p, nt, tile0 + t, 0});
                }
            } else {
                plan->n_groups_vec++;
                // a group the one-launch decode kernel can take goes to the end of the two lists
                // (the two-stage calls run the whole lists, a fused apply only their heads)
                const bool fused = fuse && n <= kExpandTok;
                std::vector<Item> &vs = fused ? vs_tail : plan->vs_items;
                std::vector<Item> &ve = fused ? ve_tail : plan->ve_items;
                if (fused) plan->vf_items.push_back(Item{off, g.rank, 0, H, pos_base, n, 0, 0});
                for (int32_t p = 0; p < n; p += shrink_tok) {
                    const int32_t nt = std::min(shrink_tok, n - p);
                    plan->max_shrink_tok = std::max(plan->max_shrink_tok, nt);
                    for (int32_t j = 0; j < g.rank; j += shrink_pages)
                        vs.push_back(Item{off, g.rank, j, std::min(shrink_pages, g.rank - j), pos_base + p, nt, 0, 0});
                }
                for (int32_t p = 0; p < n; p += kExpandTok) {
                    const int32_t nt = std::min(kExpandTok, n - p);
                    for (int32_t c = 0; c < H; c += ecols)
                        ve.push_back(Item{off, g.rank, c, std::min(ecols, H - c), pos_base + p, nt, 0, 0});
                }
            }
        }
        plan->n_vs_head = (int32_t)plan->vs_items.size();
        plan->n_ve_head = (int32_t)plan->ve_items.size();
        plan->vs_items.insert(plan->vs_items.end(), vs_tail.begin(), vs_tail.end());
        plan->ve_items.insert(plan->ve_items.end(), ve_tail.begin(), ve_tail.end());
        // longest first: the hardware hands a workgroup to a compute unit as one becomes free, so
        // with the big shares at the head of the list and the small ones at its end the launch
        // ends on every unit at about the same time
        std::stable_sort(plan->ms_items.begin(), plan->ms_items.end(), [](const MsItem &a, const MsItem &b) {
            return (int64_t)(a.ntok + a.nj) * (a.c1 - a.c0) > (int64_t)(b.ntok + b.nj) * (b.c1 - b.c0);
        });
        xcd_layout(plan->me_items, [](const Item &i) { return (int64_t)i.b * (i.ntok * 8 + i.rank * 2); }, (pool->xcd_group & 2) != 0);
        plan->T_act = (int32_t)plan->tok_idx.size();
        plan->v_stride = std::max(kRankPad, (max_rank + kRankPad - 1) / kRankPad * kRankPad);
        plan->n_rank_blocks = (plan->v_stride + kMsRanks - 1) / kMsRanks;
    } catch (const std::bad_alloc &) {
        return fail(SLORA_ENOMEM, "out of host memory while planning");
    }
    return SLORA_OK;
}

int32_t slora_plan::upload()
{
    if (!pool->dev_base) return SLORA_OK; // host-only pool: the plan stays on the host
    const size_t n_tok = tok_idx.size();
    if (n_tok == 0) return SLORA_OK;
    const size_t tok_bytes = (n_tok * sizeof(int32_t) + 63) / 64 * 64;
    const size_t bytes = tok_bytes + (ms_items.size() + mj_items.size()) * sizeof(MsItem) +
                         (vs_items.size() + ve_items.size() + me_items.size() + vf_items.size()) * sizeof(Item);
    // The image is assembled in the pinned half of a recycled buffer set and copied to the
    // device half on the pool's own upload stream: the copy runs beside whatever the caller's
    // streams are doing, and the first launch of the plan waits for it through an event.
    int32_t rc = pool->take_set(&set, bytes, bytes);
    if (rc != SLORA_OK) return rc;
    unsigned char *img = static_cast<unsigned char *>(set->h);
    std::memcpy(img, tok_idx.data(), n_tok * sizeof(int32_t));
    unsigned char *at = img + tok_bytes;
    auto put = [&](const auto &v) {
        const size_t n_bytes = v.size() * sizeof(v[0]);
        if (!v.empty()) std::memcpy(at, v.data(), n_bytes);
        at += n_bytes;
    };
    put(ms_items); // 64-byte records first: everything stays aligned to its size
    put(mj_items);
    put(vs_items);
    put(ve_items);
    put(me_items);
    put(vf_items);
    void *up_v = nullptr;
    rc = pool->uploads(&up_v);
    if (rc != SLORA_OK) {
        pool->give_set(set, nullptr);
        set = nullptr;
        return rc;
    }
    hipStream_t up = (hipStream_t)up_v;
    hipError_t e = hipMemcpyAsync(set->d, set->h, bytes, hipMemcpyHostToDevice, up);
    if (e == hipSuccess) e = hipEventRecord((hipEvent_t)set->order, up);
    if (e != hipSuccess) {
        rc = hip_fail(e, "uploading the work lists");
        pool->give_set(set, pool->upload_stream);
        set = nullptr;
        return rc;
    }
    last_stream = pool->upload_stream;
    order_recorded = true;
    d_tok_idx = (int32_t *)set->d;
    d_ms = (MsItem *)((unsigned char *)set->d + tok_bytes);
    d_mj = d_ms + ms_items.size();
    d_vs = (Item *)(d_mj + mj_items.size());
    d_ve = d_vs + vs_items.size();
    d_me = d_ve + ve_items.size();
    d_vf = d_me + me_items.size();
    return SLORA_OK;
}

void slora_plan::fill_args(MultiArgs &a, int32_t n, float *v) const
{
    const int64_t per_slot = v_slot_floats(pool->dtype);
    for (int32_t k = 0; k < n; ++k) a.v[k] = v + (int64_t)k * per_slot;
    a.vfrag_off = (int64_t)T_act * v_stride;
    a.vexp_off = a.vfrag_off + vfrag_floats(pool->dtype);
    a.part_off = a.vexp_off + vexp_floats();
}

int32_t slora_plan::enter(void *stream)
{
    if (!set || stream == last_stream) return SLORA_OK;
    hipError_t e = hipSuccess;
    if (!order_recorded) e = hipEventRecord((hipEvent_t)set->order, (hipStream_t)last_stream);
    if (e == hipSuccess) e = hipStreamWaitEvent((hipStream_t)stream, (hipEvent_t)set->order, 0);
    if (e != hipSuccess) return hip_fail(e, "ordering the plan's work between two streams");
    last_stream = stream;
    order_recorded = false;
    return SLORA_OK;
}

namespace {

int32_t check_plan(slora_plan *plan, int32_t n, const int32_t *slots)
{
    if (!plan) return fail(SLORA_EINVAL, "plan is NULL");
    if (n < 1 || n > SLORA_MAX_MULTI) return fail(SLORA_EINVAL, "n=%d must be in [1, %d]", n, SLORA_MAX_MULTI);
    if (!slots) return fail(SLORA_EINVAL, "slots is NULL");
    for (int32_t k = 0; k < n; ++k)
        if (slots[k] < 0 || slots[k] >= plan->pool->n_slots)
            return fail(SLORA_ERANGE, "slot=%d outside [0, %d)", slots[k], plan->pool->n_slots);
    if (plan->generation != plan->pool->unload_generation)
        return fail(SLORA_EBUSY, "plan is stale: an adapter was unloaded after it was built");
    if (!plan->pool->dev_base) return fail(SLORA_EHIP, "pool is host-only (dev_base == NULL)");
    return SLORA_OK;
}

// scratch: where v goes; NULL = the plan's own buffer (grown on demand)
// y != NULL: part of an apply - decode groups the plan marked for it run both stages in one
// launch here, and the two-stage launches (here and in do_expand) cover the other groups only
int32_t do_shrink(slora_plan *plan, int32_t n, const int32_t *slots, const void *const *x, void *stream,
                  float *scratch = nullptr, void *const *y = nullptr, bool y16 = false)
{
    if (!x) return fail(SLORA_EINVAL, "x is NULL");
    if (plan->T_act == 0) return SLORA_OK;
    MultiArgs a{};
    a.n = n;
    for (int32_t k = 0; k < n; ++k) {
        if (!x[k]) return fail(SLORA_EINVAL, "x[%d] is NULL", k);
        if (reinterpret_cast<uintptr_t>(x[k]) & 15) return fail(SLORA_EINVAL, "x[%d] must be 16-byte aligned", k);
        a.x[k] = x[k];
        a.slot[k] = slots[k];
    }
    DeviceScope dev(plan->pool->device);
    if (dev.status() != SLORA_OK) return dev.status();
    // the page lists of every adapter the plan names went to the device when it was built
    float *v = scratch;
    int32_t rc = SLORA_OK;
    if (!v) {
        rc = plan->pool->grow_v(plan->set, (size_t)plan->v_total_floats(n, plan->pool->dtype));
        v = plan->set->v;
    }
    if (rc == SLORA_OK) rc = plan->enter(stream);
    if (rc != SLORA_OK) return rc;
    plan->fill_args(a, n, v);
    const bool fused = y != nullptr && !plan->vf_items.empty();
    if (fused) {
        for (int32_t k = 0; k < n; ++k) a.y[k] = y[k];
        rc = launch_fused(plan, n, a, stream, y16);
        if (rc != SLORA_OK) return rc;
    }
    rc = launch_shrink(plan, n, a, stream, fused);
    if (rc == SLORA_OK) {
        plan->v_slots = n;
        plan->v_used = v;
        plan->v_complete = !fused; // after a fused apply the v of the fused groups never reached memory
    }
    return rc;
}

int32_t check_y(int32_t n, void *const *y)
{
    if (!y) return fail(SLORA_EINVAL, "y is NULL");
    for (int32_t k = 0; k < n; ++k) {
        if (!y[k]) return fail(SLORA_EINVAL, "y[%d] is NULL", k);
        if (reinterpret_cast<uintptr_t>(y[k]) & 15) return fail(SLORA_EINVAL, "y[%d] must be 16-byte aligned", k);
        for (int32_t m = 0; m < k; ++m)
            if (y[m] == y[k]) return fail(SLORA_EINVAL, "y[%d] and y[%d] are the same buffer", m, k);
    }
    return SLORA_OK;
}

int32_t do_expand(slora_plan *plan, int32_t n, const int32_t *slots, void *const *y, void *stream, bool y16,
                  bool after_fused = false)
{
    int32_t rc = check_y(n, y);
    if (rc != SLORA_OK) return rc;
    if (plan->T_act == 0) return SLORA_OK;
    MultiArgs a{};
    a.n = n;
    for (int32_t k = 0; k < n; ++k) {
        a.y[k] = y[k];
        a.slot[k] = slots[k];
    }
    if (plan->v_slots != n || !plan->v_used || (!after_fused && !plan->v_complete))
        return fail(SLORA_EINVAL, "expand of %d slot(s) needs a preceding slora_lora_shrink of %d slot(s)", n, n);
    DeviceScope dev(plan->pool->device);
    if (dev.status() != SLORA_OK) return dev.status();
    rc = plan->enter(stream);
    if (rc != SLORA_OK) return rc;
    plan->fill_args(a, n, plan->v_used);
    return launch_expand(plan, n, a, stream, y16, after_fused && !plan->vf_items.empty());
}

} // namespace

extern "C" {

int32_t slora_batch_plan(slora_pool *pool, slora_plan **out, const int32_t *token_adapter_ids, int32_t T,
                         const int32_t *seg_offsets, int32_t n_seg)
{
    clear_error();
    if (!pool || !out) return fail(SLORA_EINVAL, "NULL argument");
    *out = nullptr;
    slora_plan *p = new (std::nothrow) slora_plan;
    if (!p) return fail(SLORA_ENOMEM, "out of host memory");
    p->pool = pool;
    p->generation = pool->unload_generation;
    int32_t rc = build_plan(pool, p, token_adapter_ids, T, seg_offsets, n_seg);
    if (rc == SLORA_OK && pool->dev_base) {
        DeviceScope dev(pool->device);
        rc = dev.status();
        // page lists of adapters loaded since the last plan, then this plan's work lists
        if (rc == SLORA_OK) rc = pool->sync_device();
        if (rc == SLORA_OK) rc = p->upload();
    }
    if (rc != SLORA_OK) {
        delete p;
        return rc;
    }
    pool->live_plans++;
    *out = p;
    return SLORA_OK;
}

int32_t slora_plan_destroy(slora_plan *plan)
{
    clear_error();
    if (!plan) return SLORA_OK;
    if (plan->set) {
        // Nothing is freed and nothing is waited for: the buffers go back to the pool with an
        // event recorded behind the plan's last launch and are handed out again after it.
        DeviceScope dev(plan->pool->device);
        plan->pool->give_set(plan->set, plan->last_stream);
        plan->set = nullptr;
    }
    plan->pool->live_plans--;
    delete plan;
    return SLORA_OK;
}

int32_t slora_plan_info(const slora_plan *plan, int64_t *out, int32_t n)
{
    clear_error();
    if (!plan || !out || n < 0 || n > SLORA_PLAN_INFO_N) return fail(SLORA_EINVAL, "bad arguments");
    auto live = [](const std::vector<Item> &l) { // without the padding of the per-XCD columns
        int64_t c = 0;
        for (const Item &i : l) c += i.ntok > 0;
        return c;
    };
    const int64_t v[SLORA_PLAN_INFO_N] = {plan->T_act,
                                          plan->n_groups,
                                          plan->n_groups_vec,
                                          plan->n_groups_mfma,
                                          (int64_t)plan->vs_items.size(),
                                          (int64_t)plan->ve_items.size(),
                                          (int64_t)plan->ms_items.size(),
                                          live(plan->me_items),
                                          plan->v_stride,
                                          plan->sum_rank,
                                          plan->n_sync,
                                          plan->v_slot_floats(plan->pool->dtype) * (int64_t)sizeof(float),
                                          (int64_t)plan->vf_items.size()};
    for (int32_t k = 0; k < n; ++k) out[k] = v[k];
    return SLORA_OK;
}

int32_t slora_lora_shrink(slora_plan *plan, int32_t n, const int32_t *slots, const void *const *x, void *stream)
{
    clear_error();
    int32_t rc = check_plan(plan, n, slots);
    return rc != SLORA_OK ? rc : do_shrink(plan, n, slots, x, stream);
}

int32_t slora_lora_expand(slora_plan *plan, int32_t n, const int32_t *slots, float *const *y, void *stream)
{
    clear_error();
    int32_t rc = check_plan(plan, n, slots);
    return rc != SLORA_OK ? rc : do_expand(plan, n, slots, reinterpret_cast<void *const *>(y), stream, false);
}

int32_t slora_lora_expand_y16(slora_plan *plan, int32_t n, const int32_t *slots, void *const *y, void *stream)
{
    clear_error();
    int32_t rc = check_plan(plan, n, slots);
    return rc != SLORA_OK ? rc : do_expand(plan, n, slots, y, stream, true);
}

namespace {
int32_t apply_multi(slora_plan *plan, int32_t n, const int32_t *slots, const void *const *x, void *const *y,
                    void *stream, bool y16, bool static_scratch = false)
{
    clear_error();
    int32_t rc = check_plan(plan, n, slots);
    if (rc != SLORA_OK) return rc;
    rc = check_y(n, y); // validate the y side before the shrink is enqueued
    if (rc != SLORA_OK) return rc;
    float *scratch = nullptr;
    if (static_scratch) {
        const int64_t need = plan->v_total_floats(n, plan->pool->dtype) * (int64_t)sizeof(float);
        if (need > (int64_t)SLORA_STATIC_SCRATCH_BYTES)
            return fail(SLORA_ERANGE,
                        "this batch needs %lld bytes of scratch for %d slot(s), the static scratch holds %lld: use "
                        "fewer slots per call or slora_lora_apply_multi",
                        (long long)need, n, (long long)SLORA_STATIC_SCRATCH_BYTES);
        scratch = static_cast<float *>(plan->pool->static_scratch);
        if (!scratch) return fail(SLORA_EHIP, "the static scratch was not resolved for this pool's device");
    }
    rc = do_shrink(plan, n, slots, x, stream, scratch, y, y16);
    if (rc != SLORA_OK) return rc;
    return do_expand(plan, n, slots, y, stream, y16, true);
}
} // namespace

int32_t slora_lora_apply_multi_static(slora_plan *plan, int32_t n, const int32_t *slots, const void *const *x,
                                      float *const *y, void *stream)
{
    return apply_multi(plan, n, slots, x, reinterpret_cast<void *const *>(y), stream, false, true);
}

int32_t slora_lora_apply_multi(slora_plan *plan, int32_t n, const int32_t *slots, const void *const *x,
                               float *const *y, void *stream)
{
    return apply_multi(plan, n, slots, x, reinterpret_cast<void *const *>(y), stream, false);
}

int32_t slora_lora_apply_multi_y16(slora_plan *plan, int32_t n, const int32_t *slots, const void *const *x,
                                   void *const *y, void *stream)
{
    return apply_multi(plan, n, slots, x, y, stream, true);
}

int32_t slora_lora_apply(slora_plan *plan, int32_t slot, const void *x, float *y, void *stream)
{
    const void *xs[1] = {x};
    float *ys[1] = {y};
    return slora_lora_apply_multi(plan, 1, &slot, xs, ys, stream);
}

int32_t slora_lora_shrink_expand(slora_pool *pool, int32_t slot, const void *x, const int32_t *token_adapter_ids,
                                 const int32_t *seg_offsets, int32_t n_seg, int32_t T, float *y, void *stream)
{
    slora_plan *plan = nullptr;
    int32_t rc = slora_batch_plan(pool, &plan, token_adapter_ids, T, seg_offsets, n_seg);
    if (rc != SLORA_OK) return rc;
    rc = slora_lora_apply(plan, slot, x, y, stream);
    std::string keep = last_error_cstr();
    (void)slora_plan_destroy(plan); // the plan's buffers are recycled after the launches have run
    if (rc != SLORA_OK) fail(rc, "%s", keep.c_str());
    return rc;
}

} // extern "C"
