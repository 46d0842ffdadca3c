/*
 * slora.h - C ABI of the MI355X heterogeneous batched LoRA library.
 *
 * The library adds the low-rank term of the factored LoRA forward pass,
 *
 *      y[t,:] += (x[t,:] * A_i) * B_i ,   i = adapter of token t            (Sec. 2, Eq. 2)
 *
 * for a batch in which every token names its own adapter and adapters have different ranks
 * (Sec. 4.1, Fig. 1: the base model's xW is batched by a GEMM, the xAB term by custom kernels
 * that need no padding).  Adapter weights live in a unified pool that also holds KV-cache
 * pages: a page is one vector of H elements, a LoRA matrix of rank r occupies r pages placed
 * anywhere in the pool (Sec. 5.1, Fig. 3).  The decode path (one token per request) is the
 * paper's gather matrix-vector kernel, the prefill path (a run of tokens per request) its
 * gather matrix-matrix kernel (Sec. 5.3); here one call serves any mix of both.
 *
 * Conventions
 *   - Every function returns SLORA_OK (0) or a negative error code; nothing throws or aborts.
 *     slora_last_error() returns a thread-local message for the last failing call.
 *   - A call validates all of its arguments BEFORE it enqueues device work or changes state:
 *     after an error the pool, the adapter table and y are as they were.
 *   - "host" / "device" says where a pointer must point.  Streams are hipStream_t passed as
 *     void* (NULL = the default stream).  Device work is asynchronous on that stream unless
 *     a function says otherwise.
 *   - Storage type of pool pages and of x is IEEE binary16 or bfloat16; y and the
 *     intermediate v = x*A are fp32; all accumulation is fp32.  No alpha/r scaling is applied
 *     (Eq. 2 has none): fold any scale into B before upload.
 *     Range of v: adapter groups that run on the matrix cores (prefill segments, Sec. 5.3) hand
 *     v to the second product as 16-bit pieces whose sum is the fp32 value.  For bfloat16 pools
 *     that holds over the whole fp32 range.  For binary16 pools every token row of v is scaled
 *     by a power of two first (exponent clamped to [-24, 40]): rows whose largest |v| (per 128
 *     ranks) lies in [2^-42, 2^35) are carried to 22 bits relative to that largest value, like
 *     the fp32 sums they come from; smaller rows keep an absolute error of 2^-64; from 2^40 on
 *     the pieces overflow and y becomes inf/NaN where the vector kernels and a plain fp32
 *     evaluation would still be finite.
 *   - Page j of an adapter's A list holds column j of A (an H-vector), page j of its B list
 *     holds row j of B.  All projections map H -> H.
 *   - The pool memory is borrowed from the caller and never allocated, freed or cleared here.
 *     The library allocates only its own tables, work lists, staging buffers and the v scratch,
 *     and recycles them: a steady sequence of plan / apply / destroy (Sec. 4.1 forms a new batch
 *     every iteration) allocates nothing after the first few batches and never waits for the
 *     device.
 *   - Every call leaves the caller's current HIP device as it found it.
 *   - A handle must not be used from two threads at once.
 */
#ifndef SLORA_H
#define SLORA_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct slora_pool slora_pool; /* page ownership, adapter table, device page lists   */
typedef struct slora_plan slora_plan; /* one batch's schedule (work lists, v scratch)        */

enum { SLORA_F16 = 0, SLORA_BF16 = 1 };

enum {
    SLORA_OK = 0,
    SLORA_EINVAL = -1, /* malformed argument                                              */
    SLORA_ERANGE = -2, /* page index / slot / rank outside its range                       */
    SLORA_EBUSY = -3,  /* page already owned, adapter id already loaded, stale plan        */
    SLORA_ENOENT = -4, /* unknown adapter id                                               */
    SLORA_ESEG = -5,   /* segment offsets malformed or ids not constant inside a segment   */
    SLORA_EHIP = -6,   /* a HIP runtime call failed, or the pool has no device memory      */
    SLORA_ENOMEM = -7
};

/* Thread-local text for the most recent error returned to this thread ("" if none). */
const char *slora_last_error(void);

/*
 * Unified pool (Sec. 5.1).  dev_base: DEVICE pointer to n_pages*page_H 16-bit elements owned
 * by the caller; page p is elements [p*page_H, (p+1)*page_H).  dev_base may be NULL: the pool
 * is then host-only - ownership, adapter loading and planning work (for validation and
 * tests), every call that would touch the device returns SLORA_EHIP.
 * n_slots = number of (layer, projection) pairs every adapter carries weights for (>= 1).
 * Requirements: page_H % 8 == 0, 64 <= page_H <= 32768, 1 <= n_pages < 2^31, 0 <= max_rank <= 1024.
 * The pool uses the HIP device that is current at this call.
 */
int32_t slora_pool_init(slora_pool **out, int32_t page_H, int64_t n_pages, int32_t dtype,
                        void *dev_base, int32_t n_slots, int32_t max_rank);

/*
 * Frees the library's tables and recycled buffers after waiting for the device to go idle.
 * Plans made from the pool must be destroyed first (EBUSY).
 */
int32_t slora_pool_destroy(slora_pool *pool);

/*
 * Allocation statistics, for tests and tuning: fills out[0..n) (n <= SLORA_POOL_STATS_N) with
 *  [0] buffer sets (pinned image + device image + v scratch) ever created for plans, page
 *      writes and page-list uploads   [1] device / pinned allocations made for them and for
 *      the page-list image            [2] sets waiting to be handed out again.
 * [0] and [1] stop growing once the caller's mix of batch sizes has been seen.
 */
#define SLORA_POOL_STATS_N 3
int32_t slora_pool_stats(const slora_pool *pool, int64_t *out, int32_t n);

/*
 * Mark pages as holding KV cache (owned != 0) or release them (owned == 0).  page_idx: HOST.
 * Sec. 5.1, Fig. 3: KV-cache vectors and adapter weights are interleaved in one pool of
 * H-vector pages.
 * KV pages can never be given to an adapter; the LoRA kernels never read or write them.
 * Errors: ERANGE (index), EBUSY (page owned by an adapter, or listed twice).
 */
int32_t slora_pool_mark_kv(slora_pool *pool, const int32_t *page_idx, int64_t n, int32_t owned);

/*
 * Copy n H-vectors into the named pages: pool[page_idx[i]] = src[i*H .. (i+1)*H) (Sec. 5.1: a
 * page holds one vector of H elements, for KV cache and adapter weights alike; Sec. 5.2: adapters
 * are brought from host memory into pool pages).
 * page_idx: HOST.  src: HOST (pageable or pinned) if src_on_device == 0, else DEVICE, 16-byte
 * aligned, in the pool's storage type.  Asynchronous on `stream`: page_idx and a HOST src are
 * copied into a recycled pinned buffer before the call returns (so they may be reused at once);
 * a DEVICE src is read by a kernel on `stream` and must stay valid until the stream has run
 * it.  Ownership is not consulted (the caller also writes KV pages); only the index range is
 * checked (ERANGE).
 */
int32_t slora_pool_write_pages(slora_pool *pool, const int32_t *page_idx, int64_t n,
                               const void *src, int32_t src_on_device, void *stream);

/*
 * Make adapter `adapter_id` (any id >= 0) resident with rank `rank` (Sec. 5.1: a LoRA matrix of
 * rank r takes r pages, placed anywhere in the pool; Sec. 2: one A (H x r) and one B (r x H)
 * per adapted projection).  page_idx: HOST, n_idx =
 * n_slots*2*rank entries ordered [slot][A columns j=0..rank-1][B rows j=0..rank-1].  The
 * pages must already hold (or later receive, before the first apply) the weights.
 * rank 0 (n_idx 0) is legal: such an adapter contributes exactly nothing.
 * Errors: EINVAL (id < 0, rank < 0, n_idx mismatch), ERANGE (rank > max_rank, page index),
 * EBUSY (id already loaded; page KV-owned, owned by another adapter, or repeated).
 */
int32_t slora_adapter_load(slora_pool *pool, int32_t adapter_id, int32_t rank,
                           const int32_t *page_idx, int64_t n_idx);

/*
 * Evict the adapter (Sec. 5.1 / 5.2: adapters of finished requests make room for KV cache or
 * for other adapters): its pages become free.  Every plan built earlier becomes stale (EBUSY
 * when applied).  Launches already enqueued that use the adapter keep reading its pages and
 * page lists: the caller orders their completion before the pages are written again.
 */
int32_t slora_adapter_unload(slora_pool *pool, int32_t adapter_id);

/*
 * Page allocator of the unified pool (Sec. 5.1: KV cache and adapter weights draw H-vector pages
 * from one pool; since every request is for single pages there is no fragmentation, and the
 * two uses compete for the same free pages).  These calls let the LIBRARY choose the pages;
 * they mix freely with the calls above that name pages explicitly.
 *
 * slora_pool_free_pages: number of pages owned by nobody.
 * slora_pool_alloc_kv:   take n free pages for KV cache; their indices go to out_idx (HOST,
 *                        n entries).  Release them with slora_pool_mark_kv(..., owned = 0).
 * slora_adapter_alloc:   make the adapter resident on n_slots*2*rank pages of the library's
 *                        choice; out_idx (HOST, may be NULL) receives them in the order
 *                        [slot][A columns][B rows].  Errors as slora_adapter_load.
 * When fewer pages are free than asked for, both return SLORA_ENOMEM and take nothing: the
 * caller evicts an adapter or releases KV pages and tries again.
 */
int32_t slora_pool_free_pages(const slora_pool *pool, int64_t *out);
int32_t slora_pool_alloc_kv(slora_pool *pool, int64_t n, int32_t *out_idx);
int32_t slora_adapter_alloc(slora_pool *pool, int32_t adapter_id, int32_t rank, int32_t *out_idx);

/*
 * Fetch a resident adapter's weights into its pages, asynchronously on `stream` (Sec. 5.2: the
 * adapters of waiting requests are fetched while the running batch computes, so the copy is
 * hidden).  weights: PINNED HOST memory (hipHostMalloc; a pageable pointer is rejected with
 * EINVAL) or DEVICE memory, 16-byte aligned, n_slots*2*rank vectors of H elements of the pool's
 * storage type ordered [slot][A columns j][B rows j].  One kernel on `stream` reads the source
 * in place (over the host link for pinned memory) and scatters it to the pages: no staging
 * buffer, no synchronisation.  The source must stay valid until the stream has run the kernel;
 * an apply that uses the adapter must be ordered after it (same stream, or an event).
 */
int32_t slora_adapter_upload(slora_pool *pool, int32_t adapter_id, const void *weights, void *stream);

/*
 * Gather one paged matrix into contiguous DEVICE memory (the inverse of the paged placement of
 * Sec. 5.1, Fig. 3; what a padded batched-matmul formulation, Sec. 7.1, would have to do for
 * every token): dev_out[j*H + h] = page j of the A
 * (which = 0) or B (which = 1) list of (adapter, slot); rank*H elements, bit-exact copies.
 */
int32_t slora_adapter_gather(slora_pool *pool, int32_t adapter_id, int32_t slot, int32_t which,
                             void *dev_out, void *stream);

/*
 * Schedule a batch (Sec. 4.1: iteration-level batches mix requests of different adapters).
 * token_adapter_ids[T] and seg_offsets[n_seg+1] are HOST arrays, fully read before return.
 * A segment is one request's run of consecutive tokens: seg_offsets[0] == 0, strictly
 * increasing, seg_offsets[n_seg] == T, ids constant inside a segment (else ESEG).
 * seg_offsets == NULL: every token is its own segment (a pure decode batch); n_seg ignored.
 * id -1: the token has no adapter and its row of y is never touched.  Unknown id: ENOENT.
 * The plan groups tokens by adapter, orders groups by rank, routes small groups to the
 * matrix-vector kernels and large ones (when the batch has enough of them) to the MFMA
 * kernels, and can be applied to any slot, any number of times, until an adapter is unloaded.
 * T == 0 is legal.
 * The work lists travel to the device asynchronously on a stream the pool owns, together with
 * the page lists of adapters loaded since the previous plan; the first launch of the plan waits
 * for that copy through an event, on the device.  No host-side wait, and no allocation once
 * recycled buffers of sufficient size exist.
 */
int32_t slora_batch_plan(slora_pool *pool, slora_plan **out, const int32_t *token_adapter_ids,
                         int32_t T, const int32_t *seg_offsets, int32_t n_seg);

/*
 * End of a batch (Sec. 4.1: the batch changes every iteration).  Never waits and never frees:
 * the plan's device buffers return to the pool behind an event recorded on the stream of the
 * plan's last launch and are reused by a later plan once that event has completed.  Work the
 * plan has enqueued runs to completion as if the plan still existed.  HIP graphs that captured
 * applies of the plan must not be replayed afterwards.
 */
int32_t slora_plan_destroy(slora_plan *plan);

/*
 * Schedule statistics, for tests and tuning: fills out[0..n) (n <= SLORA_PLAN_INFO_N) with
 *  [0] tokens with an adapter of rank > 0   [1] adapter groups        [2] groups on the vector path
 *  [3] groups on the MFMA path              [4] vector shrink items   [5] vector expand items
 *  [6] MFMA shrink items                    [7] MFMA expand items     [8] v row stride (floats)
 *  [9] sum over groups of rank (pages of A read per slot)
 *  [10] MFMA shrink tiles whose H range is shared out over several workgroups
 *  [11] bytes of v scratch one slot of an apply needs
 *  [12] adapter groups an apply serves with the one-launch decode kernel
 */
#define SLORA_PLAN_INFO_N 13
int32_t slora_plan_info(const slora_plan *plan, int64_t *out, int32_t n);

/*
 * y[t,:] += (x[t,:] A_i) B_i for every token of the planned batch, weights of `slot`.
 * x: DEVICE, T*H elements of the pool's storage type, row-major.  y: DEVICE, T*H fp32,
 * row-major, updated in place.  Asynchronous on `stream`; x and y must stay valid until the
 * stream has run the work.  Rows of tokens with id -1 or a rank-0 adapter are not accessed.
 * Results are deterministic: no floating-point atomics, fixed reduction order per plan.
 * All launches of one plan share its work lists and its v scratch and therefore run in ONE
 * order: a call that names another stream than the plan's previous call makes the new stream
 * wait (on the device, through an event) for the work enqueued before.  To run projections
 * concurrently on several streams, give each stream its own plan.
 * Once a plan has been applied with n slots on a stream, further applies with at most n slots
 * on that stream allocate nothing, touch no event, and may be captured in a HIP graph; a
 * replay stays valid until the plan is destroyed or an adapter it uses is unloaded (the
 * host-side checks of this call are not part of the graph).
 */
int32_t slora_lora_apply(slora_plan *plan, int32_t slot, const void *x, float *y, void *stream);

/*
 * The same for n slots (1 <= n <= SLORA_MAX_MULTI) in one pair of launches, e.g. the q, k, v
 * projections of a layer.  slots, x, y: HOST arrays of n entries; x[k] / y[k] are DEVICE
 * pointers as in slora_lora_apply (entries of x may be equal; entries of y must not overlap).
 */
#define SLORA_MAX_MULTI 8
int32_t slora_lora_apply_multi(slora_plan *plan, int32_t n, const int32_t *slots,
                               const void *const *x, float *const *y, void *stream);

/*
 * slora_lora_apply_multi for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels,
 * same results bit for bit; the only difference is where v = x*A is kept between the two
 * launches: in a scratch array that is part of the library's code object (one copy per GPU,
 * SLORA_STATIC_SCRATCH_BYTES, held until the process ends) instead of the plan's own buffer.
 * The call makes no hipMalloc / hipFree and no other allocating call, on any path.
 * Limit: n * (tokens with an adapter * v row stride * 4 bytes + the MFMA tiles' operand
 * fragments) must fit the scratch, else SLORA_ERANGE and nothing is enqueued (slora_plan_info
 * gives tokens and stride; 8 slots of 4096 decode tokens at rank <= 128 need 16 MiB).
 * Every call on a GPU uses that GPU's one array: calls whose device work may overlap (two
 * streams, two plans, two pools) race on it - order them on one stream or by events.  Nothing
 * in the array has to be cleared between calls: the expand reads only what the shrink of the
 * same call wrote.  An expand on its own (slora_lora_expand) after this call reads the static
 * scratch too, as long as no other static call came in between.
 */
#define SLORA_STATIC_SCRATCH_BYTES (64u << 20)
int32_t slora_lora_apply_multi_static(slora_plan *plan, int32_t n, const int32_t *slots,
                                      const void *const *x, float *const *y, void *stream);

/*
 * The two stages of Eq. 2 on their own (Sec. 5.3: the custom kernels compute x*A and then
 * (x*A)*B, gathering the weights from non-contiguous pool pages without padding).  shrink
 * writes v[t,:] = x[t,:] * A_i into the plan's scratch; expand adds v[t,:] * B_i onto y[t,:].
 * An expand uses the v left by the latest shrink on the same plan with the same n.
 */
int32_t slora_lora_shrink(slora_plan *plan, int32_t n, const int32_t *slots,
                          const void *const *x, void *stream);
int32_t slora_lora_expand(slora_plan *plan, int32_t n, const int32_t *slots,
                          float *const *y, void *stream);

/*
 * 16-bit y.  The `add` node of Fig. 1 adds xAB onto the base model's xW; a serving stack keeps
 * that activation in the model's 16-bit type.  These variants take y[k] as DEVICE pointers to
 * T*H elements of the POOL'S STORAGE TYPE (binary16 or bfloat16), row-major, and compute
 *      y[t,d] = round16( fp32(y[t,d]) + sum_j v[t,j] * B_i[j,d] )
 * with the sum accumulated in fp32 exactly as in the fp32-y calls and ONE rounding to nearest,
 * ties to even, at the store.  Everything else (arguments, errors, asynchrony, rows that are
 * never touched, determinism) is as for slora_lora_apply_multi / slora_lora_expand; the shrink
 * stage is shared (slora_lora_shrink).  This halves the y traffic that dominates prefill.
 */
int32_t slora_lora_apply_multi_y16(slora_plan *plan, int32_t n, const int32_t *slots,
                                   const void *const *x, void *const *y, void *stream);
int32_t slora_lora_expand_y16(slora_plan *plan, int32_t n, const int32_t *slots,
                              void *const *y, void *stream);

/*
 * One-shot form of Eq. 2 for a batch described by its adapter ids and request segments (Sec.
 * 4.1): plan + apply(slot) + plan_destroy.  Arguments as for slora_batch_plan and
 * slora_lora_apply.  Asynchronous on `stream` like slora_lora_apply (the host arrays are fully
 * read before return); it does not wait for the device and, in the steady state, allocates
 * nothing.  A caller with several projections or layers per batch saves the scheduling work by
 * keeping one plan for all of them.
 */
int32_t slora_lora_shrink_expand(slora_pool *pool, int32_t slot, const void *x,
                                 const int32_t *token_adapter_ids, const int32_t *seg_offsets,
                                 int32_t n_seg, int32_t T, float *y, void *stream);

/*
 * Tuning knobs (affect plans made afterwards).  Keys:
 *   "mfma_min_tokens"  groups with at least this many tokens use the MFMA kernels
 *                      (default 16; 1 forces everything onto MFMA, a value > 2^30 disables it)
 *   "mfma_min_tiles"   the MFMA kernels are used only if such groups make up at least this many
 *                      32-token tiles in the batch (default 32: fewer tiles cannot fill the GPU
 *                      and run faster on the vector kernels)
 *   "mfma_split_bytes" the MFMA shrink hands the H range of a tile (up to 128 tokens x up to 128 ranks)
 *                      to several workgroups, each taking about this many bytes of x and page rows
 *                      (default 1 MiB); their partial sums are added in a fixed order by a small
 *                      second kernel
 *   "mfma_split_min_h" ... but no share of H is shorter than this many elements (default 1024, at
 *                      least 128), so that the partial sums stay small beside the rows
 *   "fuse_decode"      adapter groups of at most 4 tokens (decode) can run both stages in ONE launch, a
 *                      workgroup per group: 1 (default) when the batch has enough such groups to
 *                      fill the GPU and they average 1 MiB of pages or more, 0 never, 2 always.  Applies only (the two-stage calls
 *                      slora_lora_shrink / slora_lora_expand always use the two kernels, and an
 *                      expand on its own needs a slora_lora_shrink before it, not an apply).
 *   "shrink_pages"     pages of A per work item of the decode shrink (default 4)
 *   "upload_groups"    workgroups of slora_adapter_upload when the source is host memory (default
 *                      32: enough requests in flight to fill the host link; many more delay the
 *                      HBM traffic of kernels running on other streams)
 *   "xcd_group"        how MFMA expand items are handed to the 8 accelerator dies (one L2 each).
 *                      0 (default): round-robin.  Bit 1 (value 2): the expand list is cut into 8
 *                      contiguous, equally heavy runs, one per die, so the tiles of an adapter
 *                      share an L2 (measured 13 % slower).  Bit 0 is accepted and has no effect.
 * Results never depend on these beyond floating-point summation order.  Unknown key: EINVAL.
 */
int32_t slora_set_option(slora_pool *pool, const char *key, int64_t value);

#ifdef __cplusplus
}
#endif
#endif /* SLORA_H */
