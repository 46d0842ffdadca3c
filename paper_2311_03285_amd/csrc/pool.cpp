// Unified pool bookkeeping (Sec. 5.1): page ownership, adapter table, page-list arena and
// its device image.  Pure host logic plus a few HIP runtime calls; no kernels here.
#include <hip/hip_runtime_api.h>

#include <cstdarg>
#include <cstddef>
#include <cstdio>
#include <cstring>
#include <new>

#include "slora_internal.hpp"

namespace slora {

static thread_local std::string g_err;

int32_t fail(int32_t code, const char *fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return code;
}
void clear_error() { g_err.clear(); }
const char *last_error_cstr() { return g_err.c_str(); }

static int32_t hip_fail(hipError_t e, const char *what)
{
    return fail(SLORA_EHIP, "%s: %s", what, hipGetErrorString(e));
}

DeviceScope::DeviceScope(int device)
{
    if (device < 0) return; // host-only pool: no HIP call at all
    hipError_t e = hipGetDevice(&prev_);
    if (e == hipSuccess && prev_ != device) {
        e = hipSetDevice(device);
        switched_ = e == hipSuccess;
    }
    if (e != hipSuccess) rc_ = hip_fail(e, "selecting the pool's device");
}
DeviceScope::~DeviceScope()
{
    if (switched_) (void)hipSetDevice(prev_);
}

} // namespace slora

using namespace slora;

#define HIP_TRY(expr)                                   \
    do {                                                \
        hipError_t e_ = (expr);                         \
        if (e_ != hipSuccess) return hip_fail(e_, #expr); \
    } while (0)

// ---------------------------------------------------------------------------------------
// recycled buffer sets
// ---------------------------------------------------------------------------------------
namespace {
size_t round_up_pow2(size_t n, size_t floor)
{
    size_t c = floor;
    while (c < n) c *= 2;
    return c;
}
} // namespace

int32_t slora_pool::take_set(Buffers **out, size_t h_bytes, size_t d_bytes)
{
    *out = nullptr;
    Buffers *set = nullptr;
    // newest first: the set parked last is the most likely to be large enough
    for (size_t k = idle_sets.size(); k-- > 0;) {
        Buffers *c = idle_sets[k];
        const hipError_t q = hipEventQuery((hipEvent_t)c->order);
        if (q == hipErrorNotReady) {
            (void)hipGetLastError();
            continue; // its last user's work is still running: leave it parked
        }
        if (q != hipSuccess) return hip_fail(q, "hipEventQuery");
        set = c;
        idle_sets.erase(idle_sets.begin() + (std::ptrdiff_t)k);
        break;
    }
    if (!set) {
        set = new (std::nothrow) Buffers;
        if (!set) return fail(SLORA_ENOMEM, "out of host memory");
        hipEvent_t ev = nullptr;
        hipError_t e = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
        if (e != hipSuccess) {
            delete set;
            return hip_fail(e, "hipEventCreate");
        }
        set->order = ev;
        sets_made++;
    }
    // grow what is too small; nothing that ran on this set is still in flight, so the old
    // buffers can go at once (capacities double: a steady mix of batch sizes stops growing)
    hipError_t e = hipSuccess;
    if (set->h_cap < h_bytes) {
        if (set->h) (void)hipHostFree(set->h);
        set->h = nullptr;
        set->h_cap = 0;
        const size_t cap = round_up_pow2(h_bytes, 1 << 16);
        e = hipHostMalloc(&set->h, cap, hipHostMallocDefault);
        if (e == hipSuccess) set->h_cap = cap, device_allocs++;
    }
    if (e == hipSuccess && set->d_cap < d_bytes) {
        if (set->d) (void)hipFree(set->d);
        set->d = nullptr;
        set->d_cap = 0;
        const size_t cap = round_up_pow2(d_bytes, 1 << 16);
        e = hipMalloc(&set->d, cap);
        if (e == hipSuccess) set->d_cap = cap, device_allocs++;
    }
    if (e == hipSuccess && !set->outgrown.empty()) {
        for (void *p : set->outgrown) (void)hipFree(p);
        set->outgrown.clear();
    }
    if (e != hipSuccess) {
        idle_sets.push_back(set); // still consistent (event complete, buffers null or valid)
        return hip_fail(e, "allocating a buffer set");
    }
    *out = set;
    return SLORA_OK;
}

void slora_pool::give_set(Buffers *set, void *last_stream)
{
    if (!set) return;
    // the set may be handed out again once everything enqueued so far on its last stream has run
    (void)hipEventRecord((hipEvent_t)set->order, (hipStream_t)last_stream);
    try {
        idle_sets.push_back(set);
    } catch (const std::bad_alloc &) { // cannot park it: wait and release it instead
        (void)hipEventSynchronize((hipEvent_t)set->order);
        if (set->h) (void)hipHostFree(set->h);
        if (set->d) (void)hipFree(set->d);
        if (set->v) (void)hipFree(set->v);
        for (void *p : set->outgrown) (void)hipFree(p);
        (void)hipEventDestroy((hipEvent_t)set->order);
        delete set;
    }
}

int32_t slora_pool::grow_v(Buffers *set, size_t floats)
{
    if (floats <= set->v_cap) return SLORA_OK;
    const size_t cap = round_up_pow2(floats, 1 << 14);
    float *fresh = nullptr;
    hipError_t e = hipMalloc((void **)&fresh, cap * sizeof(float));
    if (e != hipSuccess) return hip_fail(e, "hipMalloc(v scratch)");
    device_allocs++;
    if (set->v) {
        // launches in flight, and applies captured in a HIP graph, still name the old scratch: it
        // is released when the set is next handed out (after its event) or with the pool
        try {
            set->outgrown.push_back(set->v);
        } catch (const std::bad_alloc &) {
            (void)hipFree(fresh);
            return fail(SLORA_ENOMEM, "out of host memory");
        }
    }
    set->v = fresh;
    set->v_cap = cap;
    return SLORA_OK;
}

void slora_pool::free_sets()
{
    for (Buffers *set : idle_sets) {
        if (set->h) (void)hipHostFree(set->h);
        if (set->d) (void)hipFree(set->d);
        if (set->v) (void)hipFree(set->v);
        for (void *p : set->outgrown) (void)hipFree(p);
        if (set->order) (void)hipEventDestroy((hipEvent_t)set->order);
        delete set;
    }
    idle_sets.clear();
    if (upload_stream) (void)hipStreamDestroy((hipStream_t)upload_stream);
    upload_stream = nullptr;
    if (arena_event) (void)hipEventDestroy((hipEvent_t)arena_event);
    arena_event = nullptr;
}

int32_t slora_pool::uploads(void **out)
{
    if (!upload_stream) {
        hipStream_t st = nullptr;
        // default priority; non-blocking so that it never joins the legacy default stream
        HIP_TRY(hipStreamCreateWithFlags(&st, hipStreamNonBlocking));
        upload_stream = st;
    }
    *out = upload_stream;
    return SLORA_OK;
}

// Push the page lists that changed since the last call to the device image, asynchronously on
// the upload stream (through a recycled pinned buffer); `arena_event` then marks the point
// after which the image is complete.  Plans upload their work lists on the same stream
// afterwards, so a plan's own event covers the lists too; other users wait for arena_event.
int32_t slora_pool::sync_device()
{
    if (!dev_base) return fail(SLORA_EHIP, "pool is host-only (dev_base == NULL)");
    if (dirty_hi <= dirty_lo) return SLORA_OK;
    void *up = nullptr;
    int32_t rc = uploads(&up);
    if (rc != SLORA_OK) return rc;
    const int64_t need = (int64_t)arena.size();
    if (need > d_arena_cap) {
        int64_t cap = d_arena_cap ? d_arena_cap : 4096;
        while (cap < need) cap *= 2;
        int32_t *fresh = nullptr;
        HIP_TRY(hipMalloc((void **)&fresh, (size_t)cap * sizeof(int32_t)));
        device_allocs++;
        if (d_arena) {
            // Kernels in flight, and applies captured in a HIP graph, hold the old image's address:
            // it stays allocated (and valid for every adapter loaded before this point) until
            // the pool is destroyed.  Capacities double, so the retired images add up to less
            // than the live one.
            try {
                retired_arenas.push_back(d_arena);
            } catch (const std::bad_alloc &) {
                (void)hipFree(fresh);
                return fail(SLORA_ENOMEM, "out of host memory");
            }
        }
        d_arena = fresh;
        d_arena_cap = cap;
        dirty_lo = 0;
        dirty_hi = need;
    }
    const size_t bytes = (size_t)(dirty_hi - dirty_lo) * sizeof(int32_t);
    Buffers *set = nullptr;
    rc = take_set(&set, bytes, 0);
    if (rc != SLORA_OK) return rc;
    std::memcpy(set->h, arena.data() + dirty_lo, bytes);
    hipError_t e = hipMemcpyAsync(d_arena + dirty_lo, set->h, bytes, hipMemcpyHostToDevice, (hipStream_t)up);
    if (e == hipSuccess && !arena_event) {
        hipEvent_t ev = nullptr;
        e = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
        if (e == hipSuccess) arena_event = ev;
    }
    if (e == hipSuccess) e = hipEventRecord((hipEvent_t)arena_event, (hipStream_t)up);
    give_set(set, up);
    if (e != hipSuccess) return hip_fail(e, "uploading page lists");
    dirty_lo = dirty_hi = 0;
    return SLORA_OK;
}

int32_t slora_pool::await_arena(void *stream)
{
    if (!arena_event) return SLORA_OK;
    HIP_TRY(hipStreamWaitEvent((hipStream_t)stream, (hipEvent_t)arena_event, 0));
    return SLORA_OK;
}

void slora_pool::set_state(int64_t page, uint8_t to)
{
    uint8_t &s = state[(size_t)page];
    if (s == kFree && to != kFree) n_free--;
    if (s != kFree && to == kFree) {
        n_free++;
        try {
            released.push_back((int32_t)page);
        } catch (const std::bad_alloc &) { /* the page stays free but is not handed out again */
        }
    }
    s = to;
}

int32_t slora_pool::take(int64_t n, uint8_t as, int32_t *out)
{
    if (n > n_free)
        return fail(SLORA_ENOMEM, "%lld page(s) wanted, %lld free: KV cache and adapters share the pool",
                    (long long)n, (long long)n_free);
    int64_t got = 0;
    while (got < n) {
        int64_t p = -1;
        if (!released.empty()) {
            p = released.back();
            released.pop_back();
            if (state[(size_t)p] != kFree) continue; // taken by index since it was released
        } else {
            while (fresh < n_pages && state[(size_t)fresh] != kFree) fresh++;
            if (fresh >= n_pages) break; // cannot happen while n_free is right
            p = fresh++;
        }
        state[(size_t)p] = as;
        n_free--;
        out[got++] = (int32_t)p;
    }
    if (got < n) { // give back what was taken; the count was wrong (a page could not be recorded as released)
        for (int64_t k = 0; k < got; ++k) set_state(out[k], kFree);
        return fail(SLORA_ENOMEM, "free pages could not be found");
    }
    return SLORA_OK;
}

// Record the adapter and put its page list into the arena (a freed range of the same length is
// reused).  Changes no page state; on failure nothing is recorded.
static int32_t place_list(slora_pool *pool, int32_t adapter_id, int32_t rank, const int32_t *page_idx, int64_t want)
{
    int64_t off;
    auto fl = pool->free_lists.find(want);
    try {
        if (want > 0 && fl != pool->free_lists.end() && !fl->second.empty()) {
            off = fl->second.back();
            fl->second.pop_back();
        } else {
            off = (int64_t)pool->arena.size();
            if (off + want >= (int64_t(1) << 31)) return fail(SLORA_ENOMEM, "page-list arena would exceed 2^31 entries");
            pool->arena.resize((size_t)(off + want));
        }
        pool->adapters.emplace(adapter_id, Adapter{rank, off});
    } catch (const std::bad_alloc &) {
        return fail(SLORA_ENOMEM, "out of host memory");
    }
    if (want > 0) {
        std::memcpy(pool->arena.data() + off, page_idx, (size_t)want * sizeof(int32_t));
        if (pool->dirty_hi <= pool->dirty_lo) {
            pool->dirty_lo = off;
            pool->dirty_hi = off + want;
        } else {
            if (off < pool->dirty_lo) pool->dirty_lo = off;
            if (off + want > pool->dirty_hi) pool->dirty_hi = off + want;
        }
    }
    return SLORA_OK;
}

extern "C" {

const char *slora_last_error(void) { return last_error_cstr(); }

int32_t slora_pool_init(slora_pool **out, int32_t page_H, int64_t n_pages, int32_t dtype,
                        void *dev_base, int32_t n_slots, int32_t max_rank)
{
    clear_error();
    if (!out) return fail(SLORA_EINVAL, "out is NULL");
    *out = nullptr;
    if (page_H < 64 || page_H > 32768 || page_H % 8)
        return fail(SLORA_EINVAL, "page_H=%d must be a multiple of 8 in [64, 32768]", page_H);
    if (n_pages < 1 || n_pages >= (int64_t(1) << 31))
        return fail(SLORA_EINVAL, "n_pages=%lld must be in [1, 2^31)", (long long)n_pages);
    if (dtype != SLORA_F16 && dtype != SLORA_BF16) return fail(SLORA_EINVAL, "unknown dtype %d", dtype);
    if (n_slots < 1 || n_slots > 4096) return fail(SLORA_EINVAL, "n_slots=%d must be in [1, 4096]", n_slots);
    if (max_rank < 0 || max_rank > 1024) return fail(SLORA_EINVAL, "max_rank=%d must be in [0, 1024]", max_rank);
    if (dev_base && (reinterpret_cast<uintptr_t>(dev_base) & 15))
        return fail(SLORA_EINVAL, "dev_base must be 16-byte aligned");
    int dev = -1;
    void *static_scratch = nullptr;
    if (dev_base) {
        HIP_TRY(hipGetDevice(&dev));
        // resolved here, once per GPU and with that GPU current, so that the entry point that
        // must not allocate finds the address ready
        int32_t rc = static_scratch_address(dev, &static_scratch);
        if (rc != SLORA_OK) return rc;
    }
    slora_pool *p = new (std::nothrow) slora_pool;
    if (!p) return fail(SLORA_ENOMEM, "out of host memory");
    try {
        p->state.assign((size_t)n_pages, (uint8_t)kFree);
    } catch (const std::bad_alloc &) {
        delete p;
        return fail(SLORA_ENOMEM, "out of host memory for %lld page states", (long long)n_pages);
    }
    p->H = page_H;
    p->n_pages = n_pages;
    p->dtype = dtype;
    p->dev_base = dev_base;
    p->n_slots = n_slots;
    p->max_rank = max_rank;
    p->device = dev;
    p->static_scratch = static_scratch;
    p->n_free = n_pages;
    *out = p;
    return SLORA_OK;
}

int32_t slora_pool_destroy(slora_pool *pool)
{
    clear_error();
    if (!pool) return SLORA_OK;
    if (pool->live_plans) return fail(SLORA_EBUSY, "%lld plan(s) of this pool still exist", (long long)pool->live_plans);
    if (pool->dev_base) {
        DeviceScope dev(pool->device);
        (void)hipDeviceSynchronize();
        if (pool->d_arena) (void)hipFree(pool->d_arena);
        for (int32_t *old_image : pool->retired_arenas) (void)hipFree(old_image);
        pool->free_sets();
    }
    delete pool;
    return SLORA_OK;
}

int32_t slora_pool_stats(const slora_pool *pool, int64_t *out, int32_t n)
{
    clear_error();
    if (!pool || !out || n < 0 || n > SLORA_POOL_STATS_N) return fail(SLORA_EINVAL, "bad arguments");
    const int64_t v[SLORA_POOL_STATS_N] = {pool->sets_made, pool->device_allocs, (int64_t)pool->idle_sets.size()};
    for (int32_t k = 0; k < n; ++k) out[k] = v[k];
    return SLORA_OK;
}

int32_t slora_pool_mark_kv(slora_pool *pool, const int32_t *page_idx, int64_t n, int32_t owned)
{
    clear_error();
    if (!pool) return fail(SLORA_EINVAL, "pool is NULL");
    if (n < 0 || (n > 0 && !page_idx)) return fail(SLORA_EINVAL, "bad page list");
    // validate, using a temporary mark to detect repeats, then commit
    const uint8_t kSeen = 0x80;
    int32_t rc = SLORA_OK;
    int64_t i = 0;
    for (; i < n; ++i) {
        int64_t p = page_idx[i];
        if (p < 0 || p >= pool->n_pages) {
            rc = fail(SLORA_ERANGE, "page_idx[%lld]=%lld outside [0, %lld)", (long long)i, (long long)p,
                      (long long)pool->n_pages);
            break;
        }
        uint8_t s = pool->state[p];
        if (s & kSeen) {
            rc = fail(SLORA_EBUSY, "page %lld listed twice", (long long)p);
            break;
        }
        if ((s & 0x7f) == kAdapter) {
            rc = fail(SLORA_EBUSY, "page %lld is owned by an adapter", (long long)p);
            break;
        }
        pool->state[p] = s | kSeen;
    }
    const int64_t marked = i;
    for (int64_t k = 0; k < marked; ++k) {
        uint8_t &s = pool->state[page_idx[k]];
        s &= 0x7f;
        if (rc == SLORA_OK) pool->set_state(page_idx[k], owned ? (uint8_t)kKv : (uint8_t)kFree);
    }
    return rc;
}

int32_t slora_pool_write_pages(slora_pool *pool, const int32_t *page_idx, int64_t n, const void *src,
                               int32_t src_on_device, void *stream)
{
    clear_error();
    if (!pool) return fail(SLORA_EINVAL, "pool is NULL");
    if (n < 0 || (n > 0 && (!page_idx || !src))) return fail(SLORA_EINVAL, "bad arguments");
    for (int64_t i = 0; i < n; ++i)
        if (page_idx[i] < 0 || page_idx[i] >= pool->n_pages)
            return fail(SLORA_ERANGE, "page_idx[%lld]=%d outside [0, %lld)", (long long)i, page_idx[i],
                        (long long)pool->n_pages);
    if (!pool->dev_base) return fail(SLORA_EHIP, "pool is host-only (dev_base == NULL)");
    if (n == 0) return SLORA_OK;
    DeviceScope dev(pool->device);
    if (dev.status() != SLORA_OK) return dev.status();
    hipStream_t st = (hipStream_t)stream;
    // The index list (and host-side page data) is copied into a recycled pinned buffer, from
    // there to the device with ONE asynchronous copy on `stream`, and scattered by a kernel on
    // the same stream.  The caller's arrays are free again when this call returns; the set goes
    // back to the pool and is reused after the kernel has run.
    const size_t idx_bytes = ((size_t)n * sizeof(int32_t) + 255) / 256 * 256;
    const size_t src_bytes = src_on_device ? 0 : (size_t)n * pool->H * 2;
    Buffers *set = nullptr;
    int32_t rc = pool->take_set(&set, idx_bytes + src_bytes, idx_bytes + src_bytes);
    if (rc != SLORA_OK) return rc;
    std::memcpy(set->h, page_idx, (size_t)n * sizeof(int32_t));
    if (src_bytes) std::memcpy(static_cast<unsigned char *>(set->h) + idx_bytes, src, src_bytes);
    hipError_t e = hipMemcpyAsync(set->d, set->h, idx_bytes + src_bytes, hipMemcpyHostToDevice, st);
    if (e != hipSuccess) rc = hip_fail(e, "hipMemcpyAsync(pages)");
    if (rc == SLORA_OK)
        rc = launch_write_pages(pool, static_cast<const int32_t *>(set->d), n,
                                src_on_device ? src : static_cast<const unsigned char *>(set->d) + idx_bytes, stream);
    pool->give_set(set, stream);
    return rc;
}

int32_t slora_adapter_load(slora_pool *pool, int32_t adapter_id, int32_t rank, const int32_t *page_idx,
                           int64_t n_idx)
{
    clear_error();
    if (!pool) return fail(SLORA_EINVAL, "pool is NULL");
    if (adapter_id < 0) return fail(SLORA_EINVAL, "adapter_id=%d must be >= 0", adapter_id);
    if (rank < 0) return fail(SLORA_EINVAL, "rank=%d must be >= 0", rank);
    if (rank > pool->max_rank) return fail(SLORA_ERANGE, "rank=%d exceeds max_rank=%d", rank, pool->max_rank);
    const int64_t want = (int64_t)pool->n_slots * 2 * rank;
    if (n_idx != want)
        return fail(SLORA_EINVAL, "n_idx=%lld but n_slots*2*rank=%lld", (long long)n_idx, (long long)want);
    if (want > 0 && !page_idx) return fail(SLORA_EINVAL, "page_idx is NULL");
    if (pool->adapters.count(adapter_id)) return fail(SLORA_EBUSY, "adapter %d is already loaded", adapter_id);

    const uint8_t kSeen = 0x80;
    int32_t rc = SLORA_OK;
    int64_t i = 0;
    for (; i < want; ++i) {
        int64_t p = page_idx[i];
        if (p < 0 || p >= pool->n_pages) {
            rc = fail(SLORA_ERANGE, "page_idx[%lld]=%lld outside [0, %lld)", (long long)i, (long long)p,
                      (long long)pool->n_pages);
            break;
        }
        uint8_t s = pool->state[p];
        if (s & kSeen) {
            rc = fail(SLORA_EBUSY, "page %lld appears twice in the list", (long long)p);
            break;
        }
        if (s == kKv) {
            rc = fail(SLORA_EBUSY, "page %lld holds KV cache", (long long)p);
            break;
        }
        if (s == kAdapter) {
            rc = fail(SLORA_EBUSY, "page %lld is owned by another adapter", (long long)p);
            break;
        }
        pool->state[p] = s | kSeen;
    }
    for (int64_t k = 0; k < i; ++k) pool->state[page_idx[k]] &= 0x7f;
    if (rc != SLORA_OK) return rc;

    rc = place_list(pool, adapter_id, rank, page_idx, want);
    if (rc != SLORA_OK) return rc;
    for (int64_t k = 0; k < want; ++k) pool->set_state(page_idx[k], kAdapter);
    return SLORA_OK;
}

int32_t slora_adapter_unload(slora_pool *pool, int32_t adapter_id)
{
    clear_error();
    if (!pool) return fail(SLORA_EINVAL, "pool is NULL");
    auto it = pool->adapters.find(adapter_id);
    if (it == pool->adapters.end()) return fail(SLORA_ENOENT, "adapter %d is not loaded", adapter_id);
    const int64_t len = (int64_t)pool->n_slots * 2 * it->second.rank;
    const int64_t off = it->second.arena_off;
    for (int64_t k = 0; k < len; ++k) pool->set_state(pool->arena[(size_t)(off + k)], kFree);
    if (len > 0) {
        try {
            pool->free_lists[len].push_back(off);
        } catch (const std::bad_alloc &) { /* the range is leaked inside the arena; harmless */
        }
    }
    pool->adapters.erase(it);
    pool->unload_generation++;
    return SLORA_OK;
}

int32_t slora_adapter_gather(slora_pool *pool, int32_t adapter_id, int32_t slot, int32_t which, void *dev_out,
                             void *stream)
{
    clear_error();
    if (!pool) return fail(SLORA_EINVAL, "pool is NULL");
    auto it = pool->adapters.find(adapter_id);
    if (it == pool->adapters.end()) return fail(SLORA_ENOENT, "adapter %d is not loaded", adapter_id);
    if (slot < 0 || slot >= pool->n_slots) return fail(SLORA_ERANGE, "slot=%d outside [0, %d)", slot, pool->n_slots);
    if (which != 0 && which != 1) return fail(SLORA_EINVAL, "which must be 0 (A) or 1 (B)");
    const int32_t r = it->second.rank;
    if (r > 0 && !dev_out) return fail(SLORA_EINVAL, "dev_out is NULL");
    if (r > 0 && (reinterpret_cast<uintptr_t>(dev_out) & 15)) return fail(SLORA_EINVAL, "dev_out must be 16-byte aligned");
    DeviceScope dev(pool->device);
    if (dev.status() != SLORA_OK) return dev.status();
    int32_t rc = pool->sync_device();
    if (rc == SLORA_OK) rc = pool->await_arena(stream);
    if (rc != SLORA_OK) return rc;
    if (r == 0) return SLORA_OK;
    const int64_t entry = it->second.arena_off + ((int64_t)slot * 2 + which) * r;
    return launch_gather(pool, entry, r, dev_out, stream);
}

int32_t slora_pool_free_pages(const slora_pool *pool, int64_t *out)
{
    clear_error();
    if (!pool || !out) return fail(SLORA_EINVAL, "NULL argument");
    *out = pool->n_free;
    return SLORA_OK;
}

int32_t slora_pool_alloc_kv(slora_pool *pool, int64_t n, int32_t *out_idx)
{
    clear_error();
    if (!pool) return fail(SLORA_EINVAL, "pool is NULL");
    if (n < 0 || (n > 0 && !out_idx)) return fail(SLORA_EINVAL, "bad arguments");
    return pool->take(n, kKv, out_idx);
}

int32_t slora_adapter_alloc(slora_pool *pool, int32_t adapter_id, int32_t rank, int32_t *out_idx)
{
    clear_error();
    if (!pool) return fail(SLORA_EINVAL, "pool is NULL");
    if (adapter_id < 0) return fail(SLORA_EINVAL, "adapter_id=%d must be >= 0", adapter_id);
    if (rank < 0) return fail(SLORA_EINVAL, "rank=%d must be >= 0", rank);
    if (rank > pool->max_rank) return fail(SLORA_ERANGE, "rank=%d exceeds max_rank=%d", rank, pool->max_rank);
    if (pool->adapters.count(adapter_id)) return fail(SLORA_EBUSY, "adapter %d is already loaded", adapter_id);
    const int64_t want = (int64_t)pool->n_slots * 2 * rank;
    std::vector<int32_t> pages;
    try {
        pages.resize((size_t)want);
    } catch (const std::bad_alloc &) {
        return fail(SLORA_ENOMEM, "out of host memory");
    }
    int32_t rc = pool->take(want, kAdapter, pages.data());
    if (rc != SLORA_OK) return rc;
    rc = place_list(pool, adapter_id, rank, pages.data(), want);
    if (rc != SLORA_OK) { // out of host memory for the list: the pages are free again
        std::string keep = last_error_cstr();
        for (int64_t k = 0; k < want; ++k) pool->set_state(pages[(size_t)k], kFree);
        return fail(rc, "%s", keep.c_str());
    }
    if (out_idx && want > 0) std::memcpy(out_idx, pages.data(), (size_t)want * sizeof(int32_t));
    return SLORA_OK;
}

int32_t slora_adapter_upload(slora_pool *pool, int32_t adapter_id, const void *weights, void *stream)
{
    clear_error();
    if (!pool) return fail(SLORA_EINVAL, "pool is NULL");
    auto it = pool->adapters.find(adapter_id);
    if (it == pool->adapters.end()) return fail(SLORA_ENOENT, "adapter %d is not loaded", adapter_id);
    if (!pool->dev_base) return fail(SLORA_EHIP, "pool is host-only (dev_base == NULL)");
    const int64_t n = (int64_t)pool->n_slots * 2 * it->second.rank;
    if (n == 0) return SLORA_OK;
    if (!weights) return fail(SLORA_EINVAL, "weights is NULL");
    DeviceScope dev(pool->device);
    if (dev.status() != SLORA_OK) return dev.status();
    // the copy kernel dereferences `weights` on the GPU: accept only memory the runtime knows
    // (pinned host memory or device memory), never a pageable host pointer
    hipPointerAttribute_t attr;
    hipError_t e = hipPointerGetAttributes(&attr, weights);
    if (e != hipSuccess || (attr.type != hipMemoryTypeHost && attr.type != hipMemoryTypeDevice &&
                            attr.type != hipMemoryTypeManaged) || !attr.devicePointer) {
        (void)hipGetLastError();
        return fail(SLORA_EINVAL, "weights must be pinned host memory (hipHostMalloc) or device memory");
    }
    if (reinterpret_cast<uintptr_t>(attr.devicePointer) & 15) return fail(SLORA_EINVAL, "weights must be 16-byte aligned");
    int32_t rc = pool->sync_device();
    if (rc == SLORA_OK) rc = pool->await_arena(stream);
    if (rc != SLORA_OK) return rc;
    // from host memory a few workgroups saturate the link; more only queue requests in front of
    // the HBM traffic of kernels on other streams
    const int32_t groups = attr.type == hipMemoryTypeDevice ? 0 : (int32_t)pool->upload_groups;
    return launch_write_pages(pool, pool->d_arena + it->second.arena_off, n, attr.devicePointer, stream, groups);
}

int32_t slora_set_option(slora_pool *pool, const char *key, int64_t value)
{
    clear_error();
    if (!pool || !key) return fail(SLORA_EINVAL, "NULL argument");
    if (!std::strcmp(key, "mfma_min_tokens")) {
        if (value < 1) return fail(SLORA_EINVAL, "mfma_min_tokens must be >= 1");
        pool->mfma_min_tokens = value;
        return SLORA_OK;
    }
    if (!std::strcmp(key, "mfma_min_tiles")) {
        if (value < 1) return fail(SLORA_EINVAL, "mfma_min_tiles must be >= 1");
        pool->mfma_min_tiles = value;
        return SLORA_OK;
    }
    if (!std::strcmp(key, "mfma_split_bytes")) {
        if (value < 4096) return fail(SLORA_EINVAL, "mfma_split_bytes must be >= 4096");
        pool->mfma_split_bytes = value;
        return SLORA_OK;
    }
    if (!std::strcmp(key, "mfma_split_min_h")) {
        if (value < 128) return fail(SLORA_EINVAL, "mfma_split_min_h must be >= 128");
        pool->mfma_split_min_h = value;
        return SLORA_OK;
    }
    if (!std::strcmp(key, "fuse_decode")) {
        if (value < 0 || value > 2) return fail(SLORA_EINVAL, "fuse_decode must be 0, 1 or 2");
        pool->fuse_decode = value;
        return SLORA_OK;
    }
    if (!std::strcmp(key, "shrink_pages")) {
        if (value < 1 || value > 1024) return fail(SLORA_EINVAL, "shrink_pages must be in [1, 1024]");
        pool->shrink_pages = value;
        return SLORA_OK;
    }
    if (!std::strcmp(key, "upload_groups")) {
        if (value < 1 || value > 65535) return fail(SLORA_EINVAL, "upload_groups must be in [1, 65535]");
        pool->upload_groups = value;
        return SLORA_OK;
    }
    if (!std::strcmp(key, "xcd_group")) {
        if (value < 0 || value > 3) return fail(SLORA_EINVAL, "xcd_group must be 0..3");
        pool->xcd_group = value;
        return SLORA_OK;
    }
    return fail(SLORA_EINVAL, "unknown option '%s'", key);
}

} // extern "C"
