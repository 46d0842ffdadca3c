// Host logic of the library (pool bookkeeping, scheduler, buffer recycling, argument checks)
// under AddressSanitizer / UndefinedBehaviorSanitizer, on the CPU only.
//
// pool.cpp and plan.cpp are compiled unchanged.  This file supplies (1) a stand-in for the few
// HIP runtime calls they make - "device" memory is host heap, copies are memcpy, events are
// always complete - and (2) stand-ins for the kernel launchers that do not compute anything
// but CHECK what the kernels assume about their work lists and touch every byte of scratch the
// kernels would touch, so that a list entry out of range or an undersized buffer is reported by
// the sanitizer or by an explicit check.  Then a seeded random sequence of API calls runs.
#include <hip/hip_runtime_api.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <set>
#include <vector>

#include "slora_internal.hpp"

#define REQUIRE(c)                                                          \
    do {                                                                    \
        if (!(c)) {                                                         \
            std::fprintf(stderr, "host_san: %s failed at line %d\n", #c, __LINE__); \
            std::abort();                                                   \
        }                                                                   \
    } while (0)

// ---------------------------------------------------------------------------------------------
// stand-in HIP runtime
// ---------------------------------------------------------------------------------------------
extern "C" {
hipError_t hipGetDevice(int *d) { *d = 0; return hipSuccess; }
hipError_t hipSetDevice(int) { return hipSuccess; }
hipError_t hipDeviceSynchronize(void) { return hipSuccess; }
hipError_t hipGetLastError(void) { return hipSuccess; }
const char *hipGetErrorString(hipError_t) { return "stand-in"; }
hipError_t hipMalloc(void **p, size_t n) { *p = std::malloc(n ? n : 1); return *p ? hipSuccess : hipErrorOutOfMemory; }
hipError_t hipFree(void *p) { std::free(p); return hipSuccess; }
hipError_t hipHostMalloc(void **p, size_t n, unsigned) { *p = std::malloc(n ? n : 1); return *p ? hipSuccess : hipErrorOutOfMemory; }
hipError_t hipHostFree(void *p) { std::free(p); return hipSuccess; }
hipError_t hipMemcpyAsync(void *d, const void *s, size_t n, hipMemcpyKind, hipStream_t) { std::memcpy(d, s, n); return hipSuccess; }
hipError_t hipEventCreateWithFlags(hipEvent_t *e, unsigned) { *e = (hipEvent_t)std::malloc(1); return hipSuccess; }
hipError_t hipEventDestroy(hipEvent_t e) { std::free((void *)e); return hipSuccess; }
hipError_t hipEventRecord(hipEvent_t, hipStream_t) { return hipSuccess; }
hipError_t hipEventQuery(hipEvent_t) { return hipSuccess; }
hipError_t hipEventSynchronize(hipEvent_t) { return hipSuccess; }
hipError_t hipStreamCreateWithFlags(hipStream_t *s, unsigned) { *s = (hipStream_t)std::malloc(1); return hipSuccess; }
hipError_t hipStreamDestroy(hipStream_t s) { std::free((void *)s); return hipSuccess; }
hipError_t hipStreamWaitEvent(hipStream_t, hipEvent_t, unsigned) { return hipSuccess; }
hipError_t hipPointerGetAttributes(hipPointerAttribute_t *a, const void *p)
{
    std::memset(a, 0, sizeof *a);
    a->type = hipMemoryTypeHost;
    a->devicePointer = const_cast<void *>(p);
    a->hostPointer = const_cast<void *>(p);
    return hipSuccess;
}
}

// ---------------------------------------------------------------------------------------------
// stand-in launchers: check the lists, touch the scratch
// ---------------------------------------------------------------------------------------------
namespace slora {

static std::vector<unsigned char> g_static_scratch; // exactly the size the library believes it has

int32_t static_scratch_address(int, void **out)
{
    if (g_static_scratch.empty()) g_static_scratch.resize(SLORA_STATIC_SCRATCH_BYTES);
    *out = g_static_scratch.data();
    return SLORA_OK;
}

int32_t launch_write_pages(slora_pool *pool, const int32_t *d_idx, int64_t n, const void *d_src, void *, int32_t)
{
    for (int64_t i = 0; i < n; ++i) {
        REQUIRE(d_idx[i] >= 0 && d_idx[i] < pool->n_pages);
        std::memcpy(static_cast<uint16_t *>(pool->dev_base) + (int64_t)d_idx[i] * pool->H,
                    static_cast<const uint16_t *>(d_src) + i * pool->H, (size_t)pool->H * 2);
    }
    return SLORA_OK;
}

int32_t launch_gather(slora_pool *pool, int64_t entry, int32_t rank, void *out, void *)
{
    for (int32_t j = 0; j < rank; ++j) {
        const int32_t p = pool->d_arena[entry + j];
        REQUIRE(p >= 0 && p < pool->n_pages);
        std::memcpy(static_cast<uint16_t *>(out) + (int64_t)j * pool->H,
                    static_cast<uint16_t *>(pool->dev_base) + (int64_t)p * pool->H, (size_t)pool->H * 2);
    }
    return SLORA_OK;
}

// every page number an item can reach through the device image of the arena
static void check_pages(const slora_plan *plan, int32_t arena_off, int32_t rank, int32_t slot)
{
    const slora_pool *pool = plan->pool;
    REQUIRE(arena_off >= 0 && rank > 0);
    const int64_t first = arena_off + (int64_t)slot * 2 * rank;
    REQUIRE(first + 2 * rank <= pool->d_arena_cap);
    for (int32_t j = 0; j < 2 * rank; ++j) {
        const int32_t p = pool->d_arena[first + j];
        REQUIRE(p >= 0 && p < pool->n_pages);
        REQUIRE(pool->state[(size_t)p] == kAdapter);
    }
}

static void check_tokens(const slora_plan *plan, int32_t pos0, int32_t ntok)
{
    REQUIRE(pos0 >= 0 && ntok > 0 && pos0 + ntok <= plan->T_act);
    for (int32_t t = 0; t < ntok; ++t) {
        const int32_t tok = plan->d_tok_idx[pos0 + t];
        REQUIRE(tok >= 0 && tok < plan->T);
    }
}

int32_t launch_shrink(slora_plan *plan, int32_t n, const MultiArgs &a, void *, bool heads_only)
{
    const slora_pool *pool = plan->pool;
    const int32_t np = pool->dtype == SLORA_F16 ? 2 : 3;
    const int n_gran = (pool->H + kMsGranule - 1) / kMsGranule;
    const int n_kk = plan->v_stride / 16;
    REQUIRE(a.n == n && plan->v_stride % kRankPad == 0);
    for (int32_t k = 0; k < n; ++k) {
        REQUIRE(a.x[k] && a.v[k]);
        float *v = a.v[k];
        REQUIRE(plan->n_vs_head >= 0 && (size_t)plan->n_vs_head <= plan->vs_items.size());
        for (size_t i = 0; i < (heads_only ? (size_t)plan->n_vs_head : plan->vs_items.size()); ++i) {
            const Item &it = plan->d_vs[i];
            REQUIRE(std::memcmp(&it, &plan->vs_items[i], sizeof it) == 0);
            check_pages(plan, it.arena_off, it.rank, a.slot[k]);
            check_tokens(plan, it.pos0, it.ntok);
            REQUIRE(it.ntok <= kShrinkTok && it.a >= 0 && it.b > 0 && it.b <= pool->shrink_pages && it.a + it.b <= it.rank);
            for (int32_t t = 0; t < it.ntok; ++t)
                for (int32_t j = it.a; j < it.a + it.b; ++j) v[(int64_t)(it.pos0 + t) * plan->v_stride + j] = 0.f;
        }
        uint16_t *frag = reinterpret_cast<uint16_t *>(v + a.vfrag_off);
        int8_t *vexp = reinterpret_cast<int8_t *>(v + a.vexp_off);
        float *part = v + a.part_off;
        for (size_t i = 0; i < plan->ms_items.size(); ++i) {
            const MsItem &it = plan->d_ms[i];
            REQUIRE(std::memcmp(&it, &plan->ms_items[i], sizeof it) == 0);
            check_pages(plan, it.arena_off, it.rank, a.slot[k]);
            check_tokens(plan, it.pos0, it.ntok);
            REQUIRE(it.ntok <= kMsTok && it.nj > 0 && it.nj <= kMsRanks && it.j0 % kMsRanks == 0 && it.j0 + it.nj <= it.rank);
            REQUIRE(it.c0 >= 0 && it.c0 < it.c1 && it.c1 <= n_gran && it.part >= 0 && it.part < it.n_parts);
            const int mb = (it.ntok + 31) / 32, nb = (it.nj + 31) / 32;
            REQUIRE(it.tile >= 0 && it.tile + mb <= plan->n_mfma_tiles);
            if (it.n_parts > 1) {
                REQUIRE(it.sync >= 0 && it.sync < plan->n_sync);
                REQUIRE(it.part_off >= 0 && it.part_off + (int64_t)it.n_parts * mb * nb * 1024 <= plan->part_floats);
                std::memset(part + it.part_off + (int64_t)it.part * mb * nb * 1024, 0, (size_t)mb * nb * 1024 * sizeof(float));
            }
            if (it.n_parts == 1 || it.part == it.n_parts - 1) { // the finished tile: fragments and exponents
                for (int w = 0; w < mb; ++w) {
                    for (int b = 0; b < nb; ++b)
                        for (int i2 = 0; i2 < 2; ++i2) {
                            const int kk = it.j0 / 16 + 2 * b + i2;
                            if (kk < n_kk)
                                std::memset(frag + (((int64_t)(it.tile + w) * n_kk + kk) * np) * 512, 0, (size_t)np * 1024);
                        }
                    std::memset(vexp + ((int64_t)(it.tile + w) * plan->n_rank_blocks + it.j0 / kMsRanks) * 32, 0, 32);
                }
            }
        }
        for (size_t i = 0; i < plan->mj_items.size(); ++i)
            REQUIRE(std::memcmp(&plan->d_mj[i], &plan->mj_items[i], sizeof(MsItem)) == 0);
    }
    return SLORA_OK;
}

int32_t launch_expand(slora_plan *plan, int32_t n, const MultiArgs &a, void *, bool, bool heads_only)
{
    const slora_pool *pool = plan->pool;
    REQUIRE(a.n == n);
    for (int32_t k = 0; k < n; ++k) {
        REQUIRE(a.y[k] && a.v[k]);
        REQUIRE(plan->n_ve_head >= 0 && (size_t)plan->n_ve_head <= plan->ve_items.size());
        for (size_t i = 0; i < (heads_only ? (size_t)plan->n_ve_head : plan->ve_items.size()); ++i) {
            const Item &it = plan->d_ve[i];
            REQUIRE(std::memcmp(&it, &plan->ve_items[i], sizeof it) == 0);
            check_pages(plan, it.arena_off, it.rank, a.slot[k]);
            check_tokens(plan, it.pos0, it.ntok);
            REQUIRE(it.ntok <= kExpandTok && it.a >= 0 && it.b > 0 && it.a % 8 == 0 && it.a + it.b <= pool->H);
            REQUIRE(it.b <= plan->expand_threads * 8 || plan->expand_split);
        }
        for (size_t i = 0; i < plan->me_items.size(); ++i) {
            const Item &it = plan->d_me[i];
            REQUIRE(std::memcmp(&it, &plan->me_items[i], sizeof it) == 0);
            if (it.ntok == 0) continue; // padding of a per-die column
            check_pages(plan, it.arena_off, it.rank, a.slot[k]);
            check_tokens(plan, it.pos0, it.ntok);
            REQUIRE(it.ntok <= kMfmaTok && it.a >= 0 && it.b > 0 && it.b <= kMfmaExpandCols && it.a + it.b <= pool->H);
            REQUIRE(it.tile >= 0 && it.tile < plan->n_mfma_tiles);
        }
    }
    return SLORA_OK;
}

int32_t launch_fused(slora_plan *plan, int32_t n, const MultiArgs &a, void *, bool)
{
    const slora_pool *pool = plan->pool;
    REQUIRE(a.n == n && pool->H <= 8192);
    // every fused group is a whole group of at most kExpandTok tokens, and the tails of the two
    // vector lists are exactly these groups' two-stage items
    std::set<int32_t> fused_pos;
    for (size_t i = 0; i < plan->vf_items.size(); ++i) {
        const Item &it = plan->d_vf[i];
        REQUIRE(std::memcmp(&it, &plan->vf_items[i], sizeof it) == 0);
        REQUIRE(it.ntok >= 1 && it.ntok <= kExpandTok && it.rank <= plan->v_stride);
        check_tokens(plan, it.pos0, it.ntok);
        for (int32_t k = 0; k < n; ++k) {
            REQUIRE(a.x[k] && a.y[k]);
            check_pages(plan, it.arena_off, it.rank, a.slot[k]);
        }
        fused_pos.insert(it.pos0);
    }
    for (size_t i = 0; i < plan->vs_items.size(); ++i)
        REQUIRE((fused_pos.count(plan->vs_items[i].pos0) != 0) == (i >= (size_t)plan->n_vs_head));
    for (size_t i = 0; i < plan->ve_items.size(); ++i)
        REQUIRE((fused_pos.count(plan->ve_items[i].pos0) != 0) == (i >= (size_t)plan->n_ve_head));
    return SLORA_OK;
}

} // namespace slora

// ---------------------------------------------------------------------------------------------
// driver
// ---------------------------------------------------------------------------------------------
int main(int argc, char **argv)
{
    const unsigned seed = argc > 1 ? (unsigned)std::atoi(argv[1]) : 1u;
    std::mt19937 rng(seed);
    auto rnd = [&](int lo, int hi) { return lo + (int)(rng() % (unsigned)(hi - lo + 1)); };
    long calls = 0, plans_made = 0;
    for (int round = 0; round < 12; ++round) {
        const int32_t H = 8 * rnd(8, 160);
        const int64_t n_pages = rnd(200, 3000);
        const int32_t n_slots = rnd(1, 5), max_rank = rnd(1, 300);
        const int32_t dtype = rnd(0, 1);
        std::vector<uint16_t> mem((size_t)n_pages * H, 0x3c00);
        slora_pool *pool = nullptr;
        REQUIRE(slora_pool_init(&pool, H, n_pages, dtype, mem.data(), n_slots, max_rank) == SLORA_OK);
        REQUIRE(slora_set_option(pool, "mfma_min_tokens", rnd(1, 40)) == SLORA_OK);
        REQUIRE(slora_set_option(pool, "mfma_min_tiles", rnd(1, 4)) == SLORA_OK);
        REQUIRE(slora_set_option(pool, "mfma_split_bytes", 4096 << rnd(0, 6)) == SLORA_OK);
        REQUIRE(slora_set_option(pool, "mfma_split_min_h", 128 << rnd(0, 3)) == SLORA_OK);
        REQUIRE(slora_set_option(pool, "xcd_group", rnd(0, 3)) == SLORA_OK);
        REQUIRE(slora_set_option(pool, "shrink_pages", rnd(1, 12)) == SLORA_OK);
        REQUIRE(slora_set_option(pool, "fuse_decode", rnd(0, 2)) == SLORA_OK);
        std::vector<int32_t> loaded;
        std::vector<slora_plan *> plans;
        std::vector<uint16_t> x((size_t)4096 * H, 0x3800), w;
        std::vector<float> y((size_t)SLORA_MAX_MULTI * 4096 * H, 0.f);
        for (int step = 0; step < 120; ++step, ++calls) {
            const int what = rnd(0, 9);
            if (what <= 2) { // make an adapter resident on pages of the library's choice, then fill them
                const int32_t id = rnd(0, 60), rank = rnd(0, max_rank + 2);
                std::vector<int32_t> pages((size_t)n_slots * 2 * std::max(rank, 1));
                const int32_t rc = slora_adapter_alloc(pool, id, rank, pages.data());
                if (rc == SLORA_OK) {
                    loaded.push_back(id);
                    w.assign((size_t)n_slots * 2 * rank * H + 8, 0x2e66);
                    REQUIRE(slora_adapter_upload(pool, id, w.data(), nullptr) == SLORA_OK);
                } else {
                    REQUIRE(rc == SLORA_EBUSY || rc == SLORA_ENOMEM || rc == SLORA_ERANGE);
                }
            } else if (what == 3 && !loaded.empty()) { // evict
                const size_t k = rng() % loaded.size();
                REQUIRE(slora_adapter_unload(pool, loaded[k]) == SLORA_OK);
                loaded.erase(loaded.begin() + (long)k);
            } else if (what == 4) { // KV pages come and go
                const int64_t n = rnd(0, 40);
                std::vector<int32_t> kv((size_t)std::max<int64_t>(n, 1));
                if (slora_pool_alloc_kv(pool, n, kv.data()) == SLORA_OK) {
                    std::vector<uint16_t> src((size_t)n * H, 0x7e00);
                    REQUIRE(slora_pool_write_pages(pool, kv.data(), n, src.data(), 0, nullptr) == SLORA_OK);
                    if (rnd(0, 1)) REQUIRE(slora_pool_mark_kv(pool, kv.data(), n, 0) == SLORA_OK);
                }
            } else if (what <= 7) { // a batch: prefill segments and decode tokens
                std::vector<int32_t> ids, seg{0};
                const int n_seg = rnd(0, 12);
                for (int s = 0; s < n_seg; ++s) {
                    const int32_t id = (loaded.empty() || rnd(0, 9) == 0) ? -1 : loaded[rng() % loaded.size()];
                    const int len = rnd(0, 3) ? rnd(1, 6) : rnd(20, 300);
                    if ((int)ids.size() + len > 4096) break;
                    ids.insert(ids.end(), (size_t)len, id);
                    seg.push_back((int32_t)ids.size());
                }
                slora_plan *plan = nullptr;
                const bool decode = rnd(0, 3) == 0;
                REQUIRE(slora_batch_plan(pool, &plan, ids.data(), (int32_t)ids.size(), decode ? nullptr : seg.data(),
                                         (int32_t)seg.size() - 1) == SLORA_OK);
                plans_made++;
                const int32_t n = rnd(1, SLORA_MAX_MULTI);
                int32_t slots[SLORA_MAX_MULTI];
                const void *xs[SLORA_MAX_MULTI];
                float *ys[SLORA_MAX_MULTI];
                for (int k = 0; k < n; ++k) {
                    slots[k] = rnd(0, n_slots - 1);
                    xs[k] = x.data();
                    ys[k] = y.data() + (size_t)k * 4096 * H;
                }
                const int32_t rc = rnd(0, 3) ? slora_lora_apply_multi(plan, n, slots, xs, ys, nullptr)
                                             : slora_lora_apply_multi_static(plan, n, slots, xs, ys, nullptr);
                REQUIRE(rc == SLORA_OK || rc == SLORA_ERANGE);
                int64_t info[SLORA_PLAN_INFO_N];
                REQUIRE(slora_plan_info(plan, info, SLORA_PLAN_INFO_N) == SLORA_OK);
                if (rnd(0, 2))
                    REQUIRE(slora_plan_destroy(plan) == SLORA_OK);
                else
                    plans.push_back(plan);
            } else if (what == 8 && !plans.empty()) { // an older plan again: stale after an eviction, else fine
                slora_plan *plan = plans[rng() % plans.size()];
                int32_t slot = 0;
                const void *xs[1] = {x.data()};
                float *ys[1] = {y.data()};
                const int32_t rc = slora_lora_apply_multi(plan, 1, &slot, xs, ys, nullptr);
                REQUIRE(rc == SLORA_OK || rc == SLORA_EBUSY);
            } else if (!loaded.empty()) { // gather a matrix back
                const int32_t id = loaded[rng() % loaded.size()];
                std::vector<uint16_t> out((size_t)(max_rank + 2) * H + 8);
                REQUIRE(slora_adapter_gather(pool, id, rnd(0, n_slots - 1), rnd(0, 1), out.data(), nullptr) == SLORA_OK);
            }
        }
        REQUIRE(slora_pool_destroy(pool) == SLORA_EBUSY || plans.empty());
        for (slora_plan *p : plans) REQUIRE(slora_plan_destroy(p) == SLORA_OK);
        int64_t stats[SLORA_POOL_STATS_N];
        REQUIRE(slora_pool_stats(pool, stats, SLORA_POOL_STATS_N) == SLORA_OK);
        REQUIRE(slora_pool_destroy(pool) == SLORA_OK);
    }
    std::printf("host_san OK: seed %u, %ld calls, %ld plans\n", seed, calls, plans_made);
    return 0;
}
