// Internal declarations shared by the host logic (pool, scheduler) and the kernel launchers.
#pragma once

#include <cstdint>
#include <string>
#include <unordered_map>
#include <vector>

#include "slora.h"

namespace slora {

// ---------------------------------------------------------------------------------------
// errors
// ---------------------------------------------------------------------------------------
int32_t fail(int32_t code, const char *fmt, ...) __attribute__((format(printf, 2, 3)));
void clear_error();
const char *last_error_cstr();

// ---------------------------------------------------------------------------------------
// work items (device-visible, 32 bytes)
// ---------------------------------------------------------------------------------------
// One record type serves the four work lists; `a` and `b` mean
//   vector shrink : a = first page j0 of the A list, b = number of pages
//   vector expand : a = first column (element index),  b = number of columns
//   MFMA   expand : a = first column (element index),  b = number of columns
// (the MFMA shrink has its own record, MsItem)
struct Item {
    int32_t arena_off; // adapter's first entry in the page-list arena ([slot][A r][B r])
    int32_t rank;      // r of the adapter
    int32_t a;
    int32_t b;
    int32_t pos0;      // first position in the sorted token list (also the row of v)
    int32_t ntok;      // tokens handled by this item
    int32_t tile;      // MFMA lists: number of the (adapter, 32-token) tile, shared by shrink and expand
    int32_t pad1;
};
static_assert(sizeof(Item) == 32, "Item must stay 32 bytes");

// MFMA shrink item: up to kMsTok tokens of one adapter x up to kMsRanks of its ranks x a range
// of H.  The range is the whole of H, or one of n_parts shares of it: then the workgroups of a
// tile leave their partial sums in the slot's scratch and a second kernel adds them up in the
// order of the shares.
struct MsItem {
    int32_t arena_off; // adapter's first entry in the page-list arena
    int32_t rank;      // r of the adapter
    int32_t j0, nj;    // first rank (a multiple of kMsRanks) and number of ranks
    int32_t pos0, ntok; // first position in the sorted token list, tokens
    int32_t tile;      // v tile (32 tokens) of the first token; the item covers up to 4 consecutive tiles
    int32_t c0, c1;    // granules [c0, c1) of H, kMsGranule elements each
    int32_t part, n_parts;
    int32_t sync;      // number of the tile among the plan's split tiles (-1: not split)
    int32_t part_off;  // floats from the slot's partial area to the tile's partial sums
    int32_t pad[3];
};
static_assert(sizeof(MsItem) == 64, "MsItem must stay 64 bytes");

// Per-launch arguments for up to SLORA_MAX_MULTI slots handled by one grid.
struct MultiArgs {
    const void *x[SLORA_MAX_MULTI];
    void *y[SLORA_MAX_MULTI];   // fp32 rows, or rows of the pool's storage type (16-bit y variant)
    float *v[SLORA_MAX_MULTI];
    int32_t slot[SLORA_MAX_MULTI];
    int32_t n; // slots in this launch; workgroup b handles item b / n for slot entry b % n
    int64_t vfrag_off; // floats from v[k] to the slot's v tiles in MFMA operand layout
    int64_t vexp_off;  // floats from v[k] to the per-row exponents of the tiles (binary16 pools)
    int64_t part_off;  // floats from v[k] to the partial sums of split tiles
};

// Tile constants the scheduler and the kernels must agree on.
constexpr int kShrinkTok = 4;     // tokens per vector-shrink item (x rows staged in LDS)
constexpr int kExpandTok = 4;     // tokens per vector-expand item (accumulators in registers)
constexpr int kExpandColsMax = 1024; // most columns per vector-expand item (a multiple of 512, <= 4096; measured best on cfg4: 1024)
constexpr int kMfmaTok = 32;      // tokens per v tile = per MFMA-expand item (one 32-row MFMA block)
constexpr int kMsTok = 128;       // tokens per MFMA-shrink item (one 32-row block per wavefront)
constexpr int kMsRanks = 128;     // ranks per MFMA-shrink item (up to four 32-column blocks per wavefront)
constexpr int kMsGranule = 128;   // elements of H the MFMA shrink fetches per row at a time; shares of H are whole granules
constexpr int kMfmaExpandCols = 256; // columns per MFMA-expand item (4 wavefronts x 64)
constexpr int kXcds = 8;         // accelerator dies (each with its own L2); MFMA lists are padded to this
constexpr int kRankPad = 32;      // v rows are zero-padded to a multiple of this many ranks

// ---------------------------------------------------------------------------------------
// pool
// ---------------------------------------------------------------------------------------
enum PageState : uint8_t { kFree = 0, kKv = 1, kAdapter = 2 };

struct Adapter {
    int32_t rank;
    int64_t arena_off; // into the arena, n_slots*2*rank entries
};

// A set of buffers that one plan (or one page write) uses and then hands back to the pool: a
// pinned host image, its device copy, and the v scratch.  Nothing is freed when a user lets
// go: the set waits in the pool's idle list with `order` recorded on the stream that used it
// last and is handed out again once that event has completed, so a steady stream of batches
// (Sec. 4.1: a new batch every iteration) allocates nothing and never waits for the device.
struct Buffers {
    void *h = nullptr;     // pinned host memory
    size_t h_cap = 0;
    void *d = nullptr;     // device copy of h
    size_t d_cap = 0;
    float *v = nullptr;    // device scratch for v = x*A
    size_t v_cap = 0;      // floats
    std::vector<void *> outgrown; // device buffers replaced while work that names them may be in flight
    void *order = nullptr; // hipEvent_t: last use of the set, or a hand-over point between streams
};

// Makes the pool's device current for the calling scope and restores the caller's device.
class DeviceScope {
public:
    explicit DeviceScope(int device);
    ~DeviceScope();
    int32_t status() const { return rc_; }
private:
    int prev_ = -1;
    bool switched_ = false;
    int32_t rc_ = 0;
};

} // namespace slora

struct slora_pool {
    int32_t H = 0;
    int64_t n_pages = 0;
    int32_t dtype = 0;
    void *dev_base = nullptr;
    int32_t n_slots = 0;
    int32_t max_rank = 0;
    int device = -1;

    std::vector<uint8_t> state;                       // per page
    std::unordered_map<int32_t, slora::Adapter> adapters;
    std::vector<int32_t> arena;                       // host image of all page lists
    std::unordered_map<int64_t, std::vector<int64_t>> free_lists; // length -> offsets
    int32_t *d_arena = nullptr;                       // device image
    int64_t d_arena_cap = 0;                          // entries
    std::vector<int32_t *> retired_arenas;            // outgrown device images, freed with the pool
    int64_t dirty_lo = 0, dirty_hi = 0;               // [lo, hi) not yet on the device
    // allocator: pages are handed out from a stack of released pages first (entries are checked
    // when popped: a page may have been taken by index meanwhile), then from the never-used tail
    std::vector<int32_t> released;
    int64_t fresh = 0;                                // pages >= fresh never entered `released`
    int64_t n_free = 0;
    uint64_t unload_generation = 0;
    int64_t live_plans = 0;
    int64_t mfma_min_tokens = 16;
    int64_t mfma_min_tiles = 32;
    int64_t xcd_group = 0;                            // bit 1: MFMA expand list grouped per XCD (bit 0, once the same for the shrink list, is ignored)
    int64_t upload_groups = 32;                       // workgroups of an adapter upload from host memory
    int64_t fuse_decode = 1;                          // 0: never, 1: when the batch has enough small groups, 2: always
    int64_t shrink_pages = 4;                         // pages of A per vector-shrink item (its x rows are staged once for all of them)
    int64_t mfma_split_bytes = 1 << 20;               // MFMA shrink: a tile's H range is cut into shares of about this many row bytes
    int64_t mfma_split_min_h = 1024;                  // ... but no share is shorter than this many elements of H

    // recycled buffer sets (plans, page writes) and the stream that carries work-list uploads
    std::vector<slora::Buffers *> idle_sets;
    int64_t sets_made = 0;                            // buffer sets ever allocated (steady state: constant)
    int64_t device_allocs = 0;                        // hipMalloc / hipHostMalloc calls made for them
    void *static_scratch = nullptr;                   // this GPU's copy of the library's static scratch
    void *upload_stream = nullptr;                    // hipStream_t, created on first use
    void *arena_event = nullptr;                      // hipEvent_t: the device page-list image is complete after it
    int32_t uploads(void **out);                      // the upload stream
    int32_t await_arena(void *stream);                // make `stream` wait for the latest page-list upload

    int32_t take_set(slora::Buffers **out, size_t h_bytes, size_t d_bytes); // an idle set whose last use has completed, or a new one
    void give_set(slora::Buffers *set, void *last_stream);                  // record `order` on last_stream, park the set
    int32_t grow_v(slora::Buffers *set, size_t floats);
    void free_sets();

    int32_t sync_device();                            // push dirty arena range
    void set_state(int64_t page, uint8_t to);         // ownership change with free-count / stack upkeep
    int32_t take(int64_t n, uint8_t as, int32_t *out); // n free pages -> state `as`
};

struct slora_plan {
    slora_pool *pool = nullptr;
    uint64_t generation = 0;
    int32_t T = 0;        // tokens in the batch
    int32_t T_act = 0;    // tokens that have an adapter of rank > 0
    int32_t v_stride = 0; // floats per row of v
    int32_t max_shrink_tok = 0;
    int32_t n_mfma_tiles = 0;
    int32_t expand_threads = 64; // workgroup size of the vector expand (columns per item / 8)
    int32_t expand_split = 0;    // small batch: 512-column items, ranks split over four wavefronts
    int64_t sum_rank = 0;
    int32_t n_groups = 0, n_groups_vec = 0, n_groups_mfma = 0;

    // host image
    std::vector<int32_t> tok_idx;                     // sorted position -> token index
    std::vector<slora::Item> vs_items, ve_items, me_items;
    std::vector<slora::Item> vf_items; // decode groups for the one-launch kernel (their two-stage items end vs / ve)
    int32_t n_vs_head = 0, n_ve_head = 0; // items of vs / ve that belong to other groups
    std::vector<slora::MsItem> ms_items;
    std::vector<slora::MsItem> mj_items; // one record per split tile, for the kernel that joins the shares
    int32_t ms_max_nj = 0;     // most ranks in one MFMA shrink item (sizes the kernel's LDS)
    int32_t n_sync = 0;        // split tiles
    int64_t part_floats = 0;   // partial sums of the split tiles, per slot
    int32_t n_rank_blocks = 1; // kMsRanks-blocks per row of v (exponent sets per tile)

    // device image: tok_idx and the four lists in one buffer of the plan's buffer set
    slora::Buffers *set = nullptr;
    int32_t *d_tok_idx = nullptr;
    slora::Item *d_vs = nullptr, *d_ve = nullptr, *d_me = nullptr, *d_vf = nullptr;
    slora::MsItem *d_ms = nullptr, *d_mj = nullptr;

    // scratch for v = x*A (set->v, or the library's static scratch), per slot: T_act * v_stride floats (vector path rows), n_mfma_tiles * (v_stride/16) *
    // pieces KiB of MFMA operand fragments, 32 row exponents (bytes) per tile and rank block, and the
    // partial sums of split tiles
    int64_t vfrag_floats(int32_t dtype) const
    {
        return (int64_t)n_mfma_tiles * (v_stride / 16) * (dtype == SLORA_F16 ? 2 : 3) * 256;
    }
    int64_t vexp_floats() const { return (int64_t)n_mfma_tiles * n_rank_blocks * 8; } // one byte per row
    int64_t v_slot_floats(int32_t dtype) const
    {
        return (int64_t)T_act * v_stride + vfrag_floats(dtype) + vexp_floats() + part_floats;
    }
    int64_t v_total_floats(int32_t n, int32_t dtype) const { return (int64_t)n * v_slot_floats(dtype); }
    float *v_used = nullptr; // where the latest shrink left v
    int32_t v_slots = 0;     // n of the latest shrink
    bool v_complete = false; // the latest shrink left v for every group (not so after an apply that fused decode groups)

    // Stream order.  Every launch of a plan reads its work lists and reads or writes its v, so
    // all of a plan's work is kept in ONE order: when a call names another stream than the
    // previous one, the new stream first waits for an event recorded on the old one.
    void *last_stream = nullptr; // hipStream_t of the latest upload or launch
    bool order_recorded = false; // set->order already marks the end of the work on last_stream

    int32_t upload();
    int32_t enter(void *stream);
    void fill_args(slora::MultiArgs &a, int32_t n, float *v) const;
};

namespace slora {

// scheduler (plan.cpp)
int32_t build_plan(slora_pool *pool, slora_plan *plan, const int32_t *ids, int32_t T,
                   const int32_t *seg_offsets, int32_t n_seg);

// kernel launchers (kernels.hip); all return a SLORA_* code
int32_t launch_write_pages(slora_pool *pool, const int32_t *d_idx, int64_t n, const void *d_src,
                           void *stream, int32_t max_groups = 0); // max_groups > 0 caps the grid
int32_t launch_gather(slora_pool *pool, int64_t arena_entry, int32_t rank, void *dev_out, void *stream);
int32_t static_scratch_address(int device, void **out); // `device` must be current
// heads_only: the vector lists without the groups that launch_fused has served
int32_t launch_shrink(slora_plan *plan, int32_t n, const MultiArgs &args, void *stream, bool heads_only = false);
int32_t launch_expand(slora_plan *plan, int32_t n, const MultiArgs &args, void *stream, bool y16, bool heads_only = false);
int32_t launch_fused(slora_plan *plan, int32_t n, const MultiArgs &args, void *stream, bool y16);

} // namespace slora
