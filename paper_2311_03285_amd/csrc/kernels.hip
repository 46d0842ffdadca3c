// gfx950 (CDNA4) kernels: page scatter/gather, and the shrink / expand pair of the batched
// LoRA term (Sec. 5.3: gather matrix-vector for decode, gather matrix-matrix for prefill).
//
// Data layout: pool = n_pages rows of H 16-bit elements; an adapter's page lists sit in an
// int32 arena as [slot][A columns r][B rows r]; x is T x H (16-bit), y is T x H (fp32).
// v = x*A keeps fp32 precision: the decode kernels store it as rows of `v_stride` floats indexed
// by the token's position in the plan's sorted token list, the prefill kernels as 16-bit pieces
// in MFMA operand order (see VPieces).  All byte offsets into the pool are 64-bit.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <mutex>

#include "slora_internal.hpp"

namespace slora {

namespace {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;

template <int DT>
__device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float acc)
{
    if constexpr (DT == SLORA_F16) {
        return __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, a), __builtin_bit_cast(half2_t, b), acc, false);
    } else {
        return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), acc,
                                               false);
    }
}

template <int DT>
__device__ __forceinline__ float dot8(const u32x4 &a, const u32x4 &b, float acc)
{
    acc = dot2<DT>(a.x, b.x, acc);
    acc = dot2<DT>(a.y, b.y, acc);
    acc = dot2<DT>(a.z, b.z, acc);
    acc = dot2<DT>(a.w, b.w, acc);
    return acc;
}

// the two 16-bit values packed in a dword, widened exactly to fp32
template <int DT>
__device__ __forceinline__ void widen2(uint32_t u, float &lo, float &hi)
{
    if constexpr (DT == SLORA_F16) {
        half2_t h = __builtin_bit_cast(half2_t, u);
        lo = (float)h.x;
        hi = (float)h.y;
    } else {
        lo = __uint_as_float(u << 16);
        hi = __uint_as_float(u & 0xffff0000u);
    }
}

// one fp32 value rounded to the 16-bit storage type (nearest, ties to even) and back
template <int DT>
__device__ __forceinline__ uint16_t narrow1(float f)
{
    if constexpr (DT == SLORA_F16)
        return __builtin_bit_cast(uint16_t, (_Float16)f);
    else
        return __builtin_bit_cast(uint16_t, (__bf16)f);
}
template <int DT>
__device__ __forceinline__ uint32_t narrow2(float lo, float hi)
{
    return (uint32_t)narrow1<DT>(lo) | ((uint32_t)narrow1<DT>(hi) << 16);
}
template <int DT>
__device__ __forceinline__ float widen1(uint16_t b)
{
    if constexpr (DT == SLORA_F16)
        return (float)__builtin_bit_cast(_Float16, b);
    else
        return __uint_as_float((uint32_t)b << 16);
}

// Eight consecutive elements of a row of y: fp32 (Y16 = false) or the pool's 16-bit storage
// type (Y16 = true; the sum is formed in fp32 and rounded once, to nearest even, on the way out).
// `off` is an element offset and a multiple of 8, so every access is 16-byte aligned.
template <int DT, bool Y16>
struct Y8;
template <int DT>
struct Y8<DT, false> {
    f32x4 a, b;
    __device__ __forceinline__ void load(const void *y, int64_t off)
    {
        const float *p = static_cast<const float *>(y) + off;
        a = *reinterpret_cast<const f32x4 *>(p);
        b = *reinterpret_cast<const f32x4 *>(p + 4);
    }
    __device__ __forceinline__ void add_store(void *y, int64_t off, const float (&d)[8])
    {
        float *p = static_cast<float *>(y) + off;
        a.x += d[0];
        a.y += d[1];
        a.z += d[2];
        a.w += d[3];
        b.x += d[4];
        b.y += d[5];
        b.z += d[6];
        b.w += d[7];
        *reinterpret_cast<f32x4 *>(p) = a;
        *reinterpret_cast<f32x4 *>(p + 4) = b;
    }
};
template <int DT>
struct Y8<DT, true> {
    u32x4 r;
    __device__ __forceinline__ void load(const void *y, int64_t off)
    {
        r = *reinterpret_cast<const u32x4 *>(static_cast<const uint16_t *>(y) + off);
    }
    __device__ __forceinline__ void add_store(void *y, int64_t off, const float (&d)[8])
    {
        float f[8];
        widen2<DT>(r.x, f[0], f[1]);
        widen2<DT>(r.y, f[2], f[3]);
        widen2<DT>(r.z, f[4], f[5]);
        widen2<DT>(r.w, f[6], f[7]);
        u32x4 o;
        o.x = narrow2<DT>(f[0] + d[0], f[1] + d[1]);
        o.y = narrow2<DT>(f[2] + d[2], f[3] + d[3]);
        o.z = narrow2<DT>(f[4] + d[4], f[5] + d[5]);
        o.w = narrow2<DT>(f[6] + d[6], f[7] + d[7]);
        *reinterpret_cast<u32x4 *>(static_cast<uint16_t *>(y) + off) = o;
    }
};

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, kWave);
    return v;
}

// ---------------------------------------------------------------------------------------
// page scatter / gather (exact copies)
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void write_pages_kernel(uint16_t *__restrict__ pool, const int32_t *__restrict__ idx,
                                                           const uint16_t *__restrict__ src, int H, int64_t n)
{
    // workgroups stride over the pages: a small grid bounds the requests in flight when the
    // source is host memory behind the host link
    for (int64_t i = blockIdx.x; i < n; i += gridDim.x) {
        const u32x4 *s = reinterpret_cast<const u32x4 *>(src + i * H);
        u32x4 *d = reinterpret_cast<u32x4 *>(pool + (int64_t)idx[i] * H);
        for (int c = threadIdx.x; c < H / 8; c += blockDim.x) d[c] = s[c];
    }
}

__global__ __launch_bounds__(256) void gather_pages_kernel(const uint16_t *__restrict__ pool,
                                                            const int32_t *__restrict__ list,
                                                            uint16_t *__restrict__ out, int H)
{
    const int64_t j = blockIdx.x;
    const u32x4 *s = reinterpret_cast<const u32x4 *>(pool + (int64_t)list[j] * H);
    u32x4 *d = reinterpret_cast<u32x4 *>(out + j * H);
    for (int c = threadIdx.x; c < H / 8; c += blockDim.x) d[c] = s[c];
}

// ---------------------------------------------------------------------------------------
// decode path, shrink: v[pos, j] = sum_h x[tok, h] * Apage_j[h]
//
// One workgroup (4 wavefronts) = one item = a few pages of one adapter (shrink_pages) and up to
// kShrinkTok tokens that use it.  The tokens' x rows are staged once in LDS.  Each wavefront
// streams whole pages from HBM (pages wave, wave+4, ... of the item) with 16-byte non-temporal
// loads per lane, U loads per block, two blocks in flight (the next block - possibly of the
// next page - is requested before the current one is consumed, and the very first block is
// requested before x is staged).  Blocks are dotted against the staged rows with packed
// 16-bit dot products accumulating in fp32; one 64-lane butterfly per page and token.
// ---------------------------------------------------------------------------------------
constexpr int kShrinkThreads = 256;
constexpr int kShrinkWaves = kShrinkThreads / kWave;

// The wavefront's share of `n_pages` consecutive entries of a page list (entries wave, wave + nw,
// ...), dotted against the `ntok` x rows staged in LDS; put(t, j, s) receives the finished sum
// of token t and list entry j (lane 0 only).  stage() copies the x rows to LDS and ends with a
// workgroup barrier; it runs after the first block of page data has been requested.
template <int DT, int U, class Stage, class Put>
__device__ __forceinline__ void shrink_vec_core(const int32_t *__restrict__ pa, int n_pages, int ntok, int wave, int nw,
                                                int lane, const uint16_t *__restrict__ pool, int H,
                                                const u32x4 *xs, Stage stage, Put put)
{
    const int nch = H >> 3; // 16-byte chunks per row
    const int nblk = (nch + kWave * U - 1) / (kWave * U);                           // blocks per page
    const int my_pages = n_pages > wave ? (n_pages - wave + nw - 1) / nw : 0;
    const int total = my_pages * nblk;
    const u32x4 zero = u32x4{0u, 0u, 0u, 0u};

    // block `blk` of this wavefront's page number `pg`
    auto load_block = [&](int pg, int blk, u32x4(&w)[U]) {
        const u32x4 *page = reinterpret_cast<const u32x4 *>(pool + (int64_t)pa[wave + pg * nw] * H);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int c = (blk * U + u) * kWave + lane;
            w[u] = c < nch ? __builtin_nontemporal_load(page + c) : zero;
        }
    };
    float acc[kShrinkTok];
#pragma unroll
    for (int t = 0; t < kShrinkTok; ++t) acc[t] = 0.f;
    auto consume = [&](int pg, int blk, const u32x4(&w)[U]) {
#pragma unroll
        for (int t = 0; t < kShrinkTok; ++t) {
            if (t < ntok) {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int c = (blk * U + u) * kWave + lane;
                    const u32x4 xv = c < nch ? xs[t * nch + c] : zero;
                    acc[t] = dot8<DT>(w[u], xv, acc[t]);
                }
            }
        }
        if (blk == nblk - 1) {
            const int j = wave + pg * nw;
#pragma unroll
            for (int t = 0; t < kShrinkTok; ++t) {
                if (t < ntok) {
                    const float s = wave_sum(acc[t]);
                    if (lane == 0) put(t, j, s);
                }
                acc[t] = 0.f;
            }
        }
    };

    u32x4 wa[U], wb[U];
    if (total > 0) load_block(0, 0, wa);
    stage();

    int pg = 0, blk = 0;       // position of the block held in wa
    for (int b = 0; b < total; b += 2) {
        int pg1 = pg, blk1 = blk + 1;
        if (blk1 == nblk) { blk1 = 0; ++pg1; }
        if (b + 1 < total) load_block(pg1, blk1, wb);
        consume(pg, blk, wa);
        int pg2 = pg1, blk2 = blk1 + 1;
        if (blk2 == nblk) { blk2 = 0; ++pg2; }
        if (b + 2 < total) load_block(pg2, blk2, wa);
        if (b + 1 < total) consume(pg1, blk1, wb);
        pg = pg2;
        blk = blk2;
    }
}

template <int DT, int U>
__global__ __launch_bounds__(kShrinkThreads) void shrink_vec_kernel(const Item *__restrict__ items,
                                                                     const int32_t *__restrict__ arena,
                                                                     const uint16_t *__restrict__ pool,
                                                                     const int32_t *__restrict__ tok_idx, int H,
                                                                     int v_stride, MultiArgs args)
{
    extern __shared__ u32x4 xs[]; // [ntok][H/8]
    // slots vary fastest, so workgroups are dispatched in the order of the work list (by rank)
    const int cs = blockIdx.x % args.n;
    const Item it = items[blockIdx.x / args.n];
    const uint16_t *__restrict__ x = static_cast<const uint16_t *>(args.x[cs]);
    float *__restrict__ v = args.v[cs];
    const int nch = H >> 3;
    const int tid = threadIdx.x;
    const int32_t *pa = arena + it.arena_off + (int64_t)args.slot[cs] * 2 * it.rank + it.a;
    shrink_vec_core<DT, U>(
        pa, it.b, it.ntok, tid / kWave, kShrinkWaves, tid & (kWave - 1), pool, H, xs,
        [&]() {
            for (int t = 0; t < it.ntok; ++t) {
                const u32x4 *row = reinterpret_cast<const u32x4 *>(x + (int64_t)tok_idx[it.pos0 + t] * H);
                for (int c = tid; c < nch; c += kShrinkThreads) xs[t * nch + c] = row[c];
            }
            __syncthreads();
        },
        [&](int t, int j, float s) { v[(int64_t)(it.pos0 + t) * v_stride + it.a + j] = s; });
}

// ---------------------------------------------------------------------------------------
// decode path, expand: y[tok, d] += sum_j v[pos, j] * Bpage_j[d]
//
// One workgroup = one item = a run of columns (a multiple of 512, up to 4096) of one adapter's
// B for up to kExpandTok tokens.  Each lane owns 8 adjacent columns, adjacent wavefronts own
// adjacent 1 KiB pieces of every B row, so a workgroup reads each row as one contiguous run
// of several KiB.  Rows are streamed with 16-byte non-temporal loads, U rows per block, two
// blocks in flight, widened to fp32 and accumulated as v[pos, j] * row for every token (v is
// wave-uniform and comes in through scalar loads); then one read-modify-write of y per token,
// whose loads are issued before the row loop when there are at most two tokens.
// ---------------------------------------------------------------------------------------
//
// SPLIT (small batches, where a launch has fewer workgroups than the GPU can hold): the four
// wavefronts of a workgroup own the SAME 512 columns and take every fourth block of ranks, which
// cuts the chain of dependent round trips of a high-rank item by four; their partial sums meet
// in LDS (fixed order) and wavefront 0 does the read-modify-write of y.
constexpr int kSplitWaves = 4;

template <int DT, bool Y16, int TOK, int U, bool PREFETCH_Y, bool SPLIT>
__device__ __forceinline__ void expand_vec_body(const Item &it, const int32_t *__restrict__ pb,
                                                const uint16_t *__restrict__ pool,
                                                const int32_t *__restrict__ tok_idx, int H, int v_stride,
                                                void *__restrict__ y, const float *v, int col, bool live,
                                                float *red, int v_pos0 = -1)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = SPLIT ? (int)(threadIdx.x / kWave) : 0;
    constexpr int kStep = SPLIT ? kSplitWaves : 1;
    const float *vrow = v + (int64_t)(v_pos0 < 0 ? it.pos0 : v_pos0) * v_stride; // row of v of the item's first token
    float acc[TOK][8];
#pragma unroll
    for (int t = 0; t < TOK; ++t)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[t][e] = 0.f;

    Y8<DT, Y16> yv[TOK];
    int64_t yoff[TOK];
#pragma unroll
    for (int t = 0; t < TOK; ++t) {
        yoff[t] = (int64_t)tok_idx[it.pos0 + (t < it.ntok ? t : 0)] * H + col;
        if (PREFETCH_Y && t < it.ntok && live && wave == 0) yv[t].load(y, yoff[t]);
    }

    const int col_ld = live ? col : it.a;
    // Ranks are taken in windows of 64: lane l first fetches the page index and the v values of
    // rank w0 + l (one coalesced load each); inside the window both are broadcast with readlane,
    // so the row loads of a block issue back to back with no dependent scalar loads between them.
    for (int w0 = 0; w0 < it.rank; w0 += kWave) {
        const int wr = min(kWave, it.rank - w0);
        const int pwin = lane < wr ? pb[w0 + lane] : 0;
        float vwin[TOK];
#pragma unroll
        for (int t = 0; t < TOK; ++t) vwin[t] = (t < it.ntok && lane < wr) ? vrow[t * v_stride + w0 + lane] : 0.f;

        // Straight-line blocks: rank indices beyond the window are clamped to its last rank (the
        // row is loaded again, from cache) and meet v = 0; lanes beyond the item's columns read the
        // item's first column and are dropped at the store.  No branch separates the U loads.
        const int nb = (wr + U - 1) / U;
        auto load_block = [&](int b, u32x4(&w)[U]) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int j = min(b * U + u, wr - 1);
                const int64_t page = __builtin_amdgcn_readlane(pwin, j);
                w[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(pool + page * H + col_ld));
            }
        };
        auto consume = [&](int b, const u32x4(&w)[U]) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int j = b * U + u; // < 64: nb * U <= 64
                float f[8];
                widen2<DT>(w[u].x, f[0], f[1]);
                widen2<DT>(w[u].y, f[2], f[3]);
                widen2<DT>(w[u].z, f[4], f[5]);
                widen2<DT>(w[u].w, f[6], f[7]);
#pragma unroll
                for (int t = 0; t < TOK; ++t) {
                    if (t < it.ntok) {
                        const float vv = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(vwin[t]), j));
#pragma unroll
                        for (int e = 0; e < 8; ++e) acc[t][e] = fmaf(vv, f[e], acc[t][e]);
                    }
                }
            }
        };

        u32x4 w[U];
        for (int b = wave; b < nb; b += kStep) {
            load_block(b, w);
            consume(b, w);
        }
    }

    if constexpr (SPLIT) {
        // red[wave - 1][t][e][lane]; every wavefront of the workgroup reaches both barriers
        if (wave > 0) {
#pragma unroll
            for (int t = 0; t < TOK; ++t)
#pragma unroll
                for (int e = 0; e < 8; ++e) red[(((wave - 1) * TOK + t) * 8 + e) * kWave + lane] = acc[t][e];
        }
        __syncthreads();
        if (wave > 0) return;
#pragma unroll
        for (int k = 0; k < kSplitWaves - 1; ++k)
#pragma unroll
            for (int t = 0; t < TOK; ++t)
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[t][e] += red[((k * TOK + t) * 8 + e) * kWave + lane];
    }

    if (!live) return;
#pragma unroll
    for (int t = 0; t < TOK; ++t) {
        if (t < it.ntok) {
            if (!PREFETCH_Y) yv[t].load(y, yoff[t]);
            yv[t].add_store(y, yoff[t], acc[t]);
        }
    }
}

template <int DT, bool Y16>
__global__ __launch_bounds__(512) void expand_vec_kernel(const Item *__restrict__ items,
                                                          const int32_t *__restrict__ arena,
                                                          const uint16_t *__restrict__ pool,
                                                          const int32_t *__restrict__ tok_idx, int H, int v_stride,
                                                          MultiArgs args)
{
    // slots vary fastest, so workgroups are dispatched in the order of the work list (by rank)
    const int cs = blockIdx.x % args.n;
    const Item it = items[blockIdx.x / args.n];
    const int col = it.a + threadIdx.x * 8;
    const int col_end = it.a + it.b; // <= H; both are multiples of 8
    // only WHOLE wavefronts beyond the item's columns may leave: the lanes of a wavefront exchange
    // page indices and v through readlane, so every lane of a live wavefront must stay active
    if (it.a + (int)(threadIdx.x & ~(kWave - 1)) * 8 >= col_end) return;
    const bool live = col < col_end;
    const int32_t *pb = arena + it.arena_off + (int64_t)args.slot[cs] * 2 * it.rank + it.rank;
    if (it.ntok == 1)
        expand_vec_body<DT, Y16, 1, 8, true, false>(it, pb, pool, tok_idx, H, v_stride, args.y[cs], args.v[cs], col, live, nullptr);
    else if (it.ntok == 2)
        expand_vec_body<DT, Y16, 2, 8, true, false>(it, pb, pool, tok_idx, H, v_stride, args.y[cs], args.v[cs], col, live, nullptr);
    else
        expand_vec_body<DT, Y16, kExpandTok, 8, false, false>(it, pb, pool, tok_idx, H, v_stride, args.y[cs], args.v[cs], col, live, nullptr);
}

template <int DT, bool Y16>
__global__ __launch_bounds__(kSplitWaves *kWave) void expand_vec_split_kernel(const Item *__restrict__ items,
                                                                              const int32_t *__restrict__ arena,
                                                                              const uint16_t *__restrict__ pool,
                                                                              const int32_t *__restrict__ tok_idx,
                                                                              int H, int v_stride, MultiArgs args)
{
    __shared__ float red[(kSplitWaves - 1) * kExpandTok * 8 * kWave];
    const int cs = blockIdx.x % args.n;
    const Item it = items[blockIdx.x / args.n];
    const int col = it.a + (int)(threadIdx.x & (kWave - 1)) * 8; // all four wavefronts: the same 512 columns
    const bool live = col < it.a + it.b;
    const int32_t *pb = arena + it.arena_off + (int64_t)args.slot[cs] * 2 * it.rank + it.rank;
    if (it.ntok == 1)
        expand_vec_body<DT, Y16, 1, 16, true, true>(it, pb, pool, tok_idx, H, v_stride, args.y[cs], args.v[cs], col, live, red);
    else if (it.ntok == 2)
        expand_vec_body<DT, Y16, 2, 16, true, true>(it, pb, pool, tok_idx, H, v_stride, args.y[cs], args.v[cs], col, live, red);
    else
        expand_vec_body<DT, Y16, kExpandTok, 8, false, true>(it, pb, pool, tok_idx, H, v_stride, args.y[cs], args.v[cs], col, live, red);
}


// ---------------------------------------------------------------------------------------
// decode path, both stages in ONE launch: a workgroup = one adapter group of at most kExpandTok
// tokens, one wavefront per 512 columns of H.  First the wavefronts share out the adapter's A
// pages and leave v = x*A in LDS (shrink_vec_core), then every wavefront walks the B pages for
// its own columns (expand_vec_body) and updates y.  v never leaves the compute unit, x is staged
// once per group instead of once per four pages, and a decode step is one kernel instead of
// two dependent ones (each of which spends its first microseconds waiting for work items,
// page lists and the first pages).  Used when a batch has enough such groups to fill the GPU
// with whole-group workgroups (the scheduler decides); results are bit-identical to the two
// kernels' - the same sums in the same order.
// ---------------------------------------------------------------------------------------
template <int DT, bool Y16, int U>
__global__ __launch_bounds__(1024) void lora_vec_fused_kernel(const Item *__restrict__ items,
                                                               const int32_t *__restrict__ arena,
                                                               const uint16_t *__restrict__ pool,
                                                               const int32_t *__restrict__ tok_idx, int H,
                                                               int v_pad, MultiArgs args)
{
    extern __shared__ u32x4 smem[]; // x rows [kExpandTok][H/8], then v [kExpandTok][v_pad] floats
    const int cs = blockIdx.x % args.n;
    const Item it = items[blockIdx.x / args.n];
    const uint16_t *__restrict__ x = static_cast<const uint16_t *>(args.x[cs]);
    const int nch = H >> 3;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    const int nw = blockDim.x / kWave;
    float *vl = reinterpret_cast<float *>(smem + (size_t)kExpandTok * nch);
    const int32_t *pa = arena + it.arena_off + (int64_t)args.slot[cs] * 2 * it.rank;
    shrink_vec_core<DT, U>(
        pa, it.rank, it.ntok, wave, nw, lane, pool, H, smem,
        [&]() {
            for (int t = 0; t < it.ntok; ++t) {
                const u32x4 *row = reinterpret_cast<const u32x4 *>(x + (int64_t)tok_idx[it.pos0 + t] * H);
                for (int c = tid; c < nch; c += (int)blockDim.x) smem[t * nch + c] = row[c];
            }
            __syncthreads();
        },
        [&](int t, int j, float s) { vl[t * v_pad + j] = s; });
    __syncthreads();
    // expand: 512-column strips wave, wave + nw, ... (one strip per wavefront for H <= 8192)
    const int32_t *pb = pa + it.rank;
    for (int c0 = wave * 512; c0 < H; c0 += nw * 512) {
        const int col = c0 + lane * 8;
        const bool live = col < H;
        Item strip = it;
        strip.a = c0;   // lanes beyond H read the strip's first column and are dropped at the store
        if (it.ntok == 1)
            expand_vec_body<DT, Y16, 1, 8, true, false>(strip, pb, pool, tok_idx, H, v_pad, args.y[cs], vl, col, live, nullptr, 0);
        else if (it.ntok == 2)
            expand_vec_body<DT, Y16, 2, 8, true, false>(strip, pb, pool, tok_idx, H, v_pad, args.y[cs], vl, col, live, nullptr, 0);
        else
            expand_vec_body<DT, Y16, kExpandTok, 8, false, false>(strip, pb, pool, tok_idx, H, v_pad, args.y[cs], vl, col, live, nullptr, 0);
    }
}

// ---------------------------------------------------------------------------------------
// prefill path (MFMA).  Matrix blocks are 32 x 32 with 16 k-values per instruction
// (v_mfma_f32_32x32x16_{f16,bf16}): lane l supplies, for row/column l % 32, the 8 k-values
// 8*(l / 32) .. +7 of both operands, and receives D[8*(v/4) + 4*(l/32) + v%4][l % 32] in
// accumulator register v (0..15).
// ---------------------------------------------------------------------------------------
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

template <int DT>
__device__ __forceinline__ f32x16 mfma32(const u32x4 &a, const u32x4 &b, const f32x16 &c)
{
    if constexpr (DT == SLORA_F16)
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0,
                                                      0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c,
                                                       0, 0, 0);
}

// Workgroup -> (item, slot) for the MFMA work lists.  The scheduler lays these lists out in rows
// of kXcds items, column k holding work of the k-th share of the batch; workgroups are handed
// to the 8 XCDs round-robin by their linear id, so making the item's column the fastest-varying
// part of the id keeps every share on one XCD (all tiles of an adapter then find its pages in
// that XCD's L2).  Within a row the slots follow one another.
__device__ __forceinline__ int mfma_item_of(unsigned bid, int n)
{
    const unsigned per_row = kXcds * (unsigned)n;
    return (int)((bid / per_row) * kXcds + (bid % kXcds));
}
__device__ __forceinline__ int mfma_slot_of(unsigned bid, int n)
{
    return (int)((bid % (kXcds * (unsigned)n)) / kXcds);
}

// accumulator register v of lane `lane` holds this row of the 32 x 32 block
__device__ __forceinline__ int mfma_row(int v, int lane) { return 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3); }

// v = x*A of the MFMA path is handed from shrink to expand already in the layout of the expand's
// first MFMA operand, split into 16-bit pieces whose sum is the fp32 value (so nothing is lost to
// the operand format): hi + lo for binary16 (22+ bits), hi + mid + lo by truncation for bfloat16
// (exactly 24 bits).  One fragment = 64 lanes x 8 values (1 KiB) = the operand of one MFMA:
// tokens 0..31 of the tile x ranks 16*kk .. 16*kk+15, lane = token + 32 * ((rank % 16) / 8).
// Fragments are ordered [tile][kk][piece]; the expand reads each with one coalesced 16-byte load
// per lane and does no conversion work.
template <int DT>
struct VPieces {
    static constexpr int N = DT == SLORA_F16 ? 2 : 3;
};
__device__ __forceinline__ int64_t vfrag_index(int tile, int kk, int piece, int n_kk, int n_piece)
{
    return (((int64_t)tile * n_kk + kk) * n_piece + piece) * (kWave * 8);
}
// eight consecutive ranks of one token -> the 16-bit pieces whose sum is the fp32 value, packed as
// the 16 bytes a lane owns in each piece's fragment
template <int DT>
__device__ __forceinline__ void split_pieces(const float (&f)[8], u32x4 (&piece)[VPieces<DT>::N])
{
    uint16_t h[VPieces<DT>::N][8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        if constexpr (DT == SLORA_F16) {
            const _Float16 a = (_Float16)f[e];
            const _Float16 b = (_Float16)(f[e] - (float)a);
            h[0][e] = __builtin_bit_cast(uint16_t, a);
            h[1][e] = __builtin_bit_cast(uint16_t, b);
        } else {
            const uint32_t hi = __float_as_uint(f[e]) & 0xffff0000u;
            const float r1 = f[e] - __uint_as_float(hi);
            const uint32_t mid = __float_as_uint(r1) & 0xffff0000u;
            const float r2 = r1 - __uint_as_float(mid);
            h[0][e] = (uint16_t)(hi >> 16);
            h[1][e] = (uint16_t)(mid >> 16);
            h[2][e] = (uint16_t)(__float_as_uint(r2) >> 16);
        }
    }
#pragma unroll
    for (int p = 0; p < VPieces<DT>::N; ++p)
#pragma unroll
        for (int k = 0; k < 4; ++k) piece[p][k] = (uint32_t)h[p][2 * k] | ((uint32_t)h[p][2 * k + 1] << 16);
}

// ---------------------------------------------------------------------------------------
// prefill shrink: V[pos, j] = sum_h x[tok, h] * Apage_j[h] for up to 128 tokens of one adapter
// (MB = 2 or 4 blocks of 32 rows, one per wavefront), up to 128 of its ranks (NB = 1, 2 or 4
// blocks of 32) and a range of H.
//
// An LDS-tiled product with the second operand gathered through the page list.  The range of H
// is walked in chunks of 64 elements.  Per chunk the workgroup copies the x rows and the page
// rows (128 bytes of each) into LDS; the rows are fetched 256 bytes at a time with coalesced
// 16-byte loads through a register ring that keeps two such granules in flight.  LDS rows are
// padded by 16 bytes; wavefront w owns token block w, reads its operands in MFMA layout with
// 16-byte LDS loads and accumulates 32 x 32 tiles for all rank blocks, so no sum across
// wavefronts is needed.  Large tiles (128 tokens share every page row) keep the pages from
// being fetched once per 32 or 64 tokens.
//
// A workgroup streams its rows at a rate set by the loads it keeps in flight, so the scheduler
// cuts the H range of a tile into n_parts shares, one workgroup each.  A share leaves its
// partial sums (fp32) in the slot's scratch; a second, small kernel (join_shares_kernel, one
// workgroup per split tile) adds them up in the order of their numbers.  The kernel boundary
// is the only synchronisation: arrival counters with device-wide fences inside the shrink were
// tried and cost more than the extra launch (a fence per workgroup writes back and invalidates
// the die's whole L2: cfg3's shrink went from 77 us unsplit to 93 us with 168 shares).
//
// The finished tile goes to the expand as MFMA operand fragments (see VPieces).  For binary16
// pools every token row is first scaled by a power of two, 2^e, that puts its largest |v| into
// [2^10, 2^11): the hi piece then holds 11 bits and the lo piece 11 more whatever the magnitude
// of v (row maxima in [2^-42, 2^35); the pieces overflow from 2^40 on).  e (clamped to [-24, 40]) is left
// beside the fragments; the expand scales its accumulators by 2^e and back.
// Token rows beyond the item and ranks beyond the adapter's are read from a valid row instead;
// their results are not stored, or stored as zero (ranks up to the next multiple of 32, so the
// expand can read whole blocks).
// ---------------------------------------------------------------------------------------
constexpr int kMfmaThreads = 256;
constexpr int kMsChunk = kMsGranule / 2;             // elements of H per LDS chunk
constexpr int kMsRowBytes = kMsChunk * 2;            // bytes of one row per chunk
constexpr int kMsGranuleBytes = kMsGranule * 2;      // bytes of one row fetched at a time
constexpr int kMsLdsRow = kMsRowBytes + 16;          // padded LDS row
constexpr int kRing = 2;                             // granules in flight
constexpr int kMsRowsPerPass = kMfmaThreads / 8;     // rows covered by one load per thread
constexpr int kEpiStride = 36;                       // floats per row of a wavefront's 32 x 32 staging tile
constexpr int kExpMin = -24, kExpMax = 40;           // range of the row exponents of binary16 pools
static_assert(kMsRowsPerPass == 32 && kMsTok == 128 && kMsRanks == 128, "copy duty and tile shape are tied");

__device__ __forceinline__ float pow2f(int e) { return __uint_as_float((uint32_t)(e + 127) << 23); }

// Partial sums of a split tile: [share][token block][rank block][octet pair i][lane][8 floats];
// lane l holds token l % 32 of its wavefront's block and the rank octets l / 32 + 2 i.
template <int NB>
__device__ __forceinline__ void store_share(const MsItem &it, int wave, int lane, const float (&val)[NB][2][8],
                                            float *__restrict__ partial)
{
    const int mb_act = (it.ntok + 31) >> 5, nb_act = (it.nj + 31) >> 5;
    const int64_t blk = (int64_t)mb_act * nb_act * 1024;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        if (nb < nb_act) {
            float *dst = partial + it.part * blk + (int64_t)(wave * nb_act + nb) * 1024 + lane * 8;
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                *reinterpret_cast<f32x4 *>(dst + i * 512) = f32x4{val[nb][i][0], val[nb][i][1], val[nb][i][2], val[nb][i][3]};
                *reinterpret_cast<f32x4 *>(dst + i * 512 + 4) =
                    f32x4{val[nb][i][4], val[nb][i][5], val[nb][i][6], val[nb][i][7]};
            }
        }
    }
}

// Exponent e of the power of two that scales a token row of a binary16 pool: the row's largest
// |v| lands in [2^10, 2^11).  Zero, subnormal, infinite and NaN maxima get e = 0.
__device__ __forceinline__ int row_exponent(float vmax)
{
    const int be = (int)((__float_as_uint(vmax) >> 23) & 0xffu); // biased exponent of the row maximum
    if (be == 0 || be == 255) return 0;
    return min(max(10 - (be - 127), kExpMin), kExpMax);
}

// Ranks beyond the adapter's become zero; returns the largest |value| this lane holds in the block.
__device__ __forceinline__ float mask_block(const MsItem &it, int nb, int q, float (&val)[2][8])
{
    float vmax = 0.f;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int jn = nb * 32 + (q + 2 * i) * 8 + e;
            const float f = jn < it.nj ? val[i][e] : 0.f;
            val[i][e] = f;
            vmax = fmaxf(vmax, fabsf(f));
        }
    return vmax;
}

// One 32-token x 32-rank block of finished sums -> the two operand fragments it fills (lane l:
// token l % 32, rank octets l / 32 and l / 32 + 2), scaled by `sc` first.
template <int DT>
__device__ __forceinline__ void store_block(const MsItem &it, int tile, int nb, int lane, const float (&val)[2][8],
                                            float sc, int v_stride, uint16_t *__restrict__ vfrag)
{
    constexpr int NP = VPieces<DT>::N;
    const int n_kk = v_stride >> 4;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int kk = (it.j0 >> 4) + 2 * nb + i;
        if (kk < n_kk) {
            float f[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) f[k] = DT == SLORA_F16 ? val[i][k] * sc : val[i][k];
            uint16_t *dst = vfrag + vfrag_index(tile, kk, 0, n_kk, NP) + lane * 8;
            u32x4 piece[NP];
            split_pieces<DT>(f, piece);
#pragma unroll
            for (int p = 0; p < NP; ++p) *reinterpret_cast<u32x4 *>(dst + p * (kWave * 8)) = piece[p];
        }
    }
}

// Row exponents are kept as signed bytes, 32 per (v tile, rank block), ordered so that the 16
// exponents a lane of the expand needs - accumulator register 4 g + k of lane half q holds row
// 8 g + 4 q + k - are the 16 consecutive bytes q * 16 + g * 4 + k: one 16-byte load.
__device__ __forceinline__ int8_t *vexp_row(int8_t *vexp, const MsItem &it, int tile, int v_stride, int row)
{
    const int n_rb = (v_stride + kMsRanks - 1) / kMsRanks;
    const int g = row >> 3, qq = (row >> 2) & 1, k = row & 3;
    return vexp + ((int64_t)tile * n_rb + it.j0 / kMsRanks) * 32 + qq * 16 + g * 4 + k;
}

// The finished sums of one token block (this wavefront's), all rank blocks -> operand fragments.
template <int DT, int NB>
__device__ __forceinline__ void finish_tile(const MsItem &it, int wave, int lane, float (&val)[NB][2][8], int v_stride,
                                            uint16_t *__restrict__ vfrag, int8_t *__restrict__ vexp)
{
    const int row = lane & 31, q = lane >> 5;
    const int nb_act = (it.nj + 31) >> 5;
    const bool token_ok = wave * 32 + row < it.ntok;
    float vmax = 0.f;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
        if (nb < nb_act) vmax = fmaxf(vmax, mask_block(it, nb, q, val[nb]));
    float sc = 1.f;
    if constexpr (DT == SLORA_F16) {
        vmax = fmaxf(vmax, __shfl_xor(vmax, 32, kWave)); // the other half of the token's ranks
        const int e = row_exponent(vmax);
        sc = pow2f(e);
        if (q == 0) *vexp_row(vexp, it, it.tile + wave, v_stride, row) = (int8_t)(token_ok ? e : 0);
    }
    if (!token_ok) return;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
        if (nb < nb_act) store_block<DT>(it, it.tile + wave, nb, lane, val[nb], sc, v_stride, vfrag);
}

template <int DT, int NB, int MB>
__device__ __forceinline__ void shrink_mfma_tile(const MsItem &it, const int32_t *__restrict__ pa,
                                                 const unsigned char *__restrict__ x,
                                                 const uint16_t *__restrict__ pool,
                                                 const int32_t *__restrict__ tok_idx, int H, int v_stride,
                                                 uint16_t *__restrict__ vfrag, int8_t *__restrict__ vexp,
                                                 float *__restrict__ partial, unsigned char *lds, int args_n)
{
    constexpr int kLoads = MB + NB;                 // 16-byte loads per thread and chunk
    constexpr int kRows = 32 * (MB + NB);           // LDS rows of one buffer
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    const int row = lane & 31;
    const int q = lane >> 5;
    const int64_t row_bytes = (int64_t)H * 2;

    // ---- copy duty of this thread: byte column cb of LDS rows r8 + 32*i (x rows, then pages)
    const int r8 = tid >> 3;
    const int cb = (tid & 7) * 16;
    const unsigned char *src[kLoads];
#pragma unroll
    for (int i = 0; i < MB; ++i) {
        const int r = r8 + kMsRowsPerPass * i;
        src[i] = x + (int64_t)tok_idx[it.pos0 + (r < it.ntok ? r : 0)] * row_bytes;
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int j = r8 + kMsRowsPerPass * i;
        src[MB + i] = reinterpret_cast<const unsigned char *>(pool) + (int64_t)pa[j < it.nj ? j : 0] * row_bytes;
    }
    const int n_gran = it.c1 - it.c0;

    // Memory is read in granules of 256 bytes per row (two LDS chunks): a thread fetches the two
    // 16-byte pieces cb and cb + 128 of a granule back to back, so the two 128-byte lines of a
    // granule are requested together (128-byte pieces fetched a chunk apart ran at two thirds of
    // the rate).
    struct Regs {
        u32x4 w[2][kLoads];
    };
    // Every workgroup starts its sweep over the share at another granule and wraps around: tiles
    // launched together would otherwise walk H in lockstep, all of them asking the same few memory
    // channels for the same column offset of their rows at the same time (a load-only probe of
    // this access pattern: 4.5 TB/s in lockstep, 5.5 TB/s with staggered starts).  The order of a
    // sum over H changes with it, its value only in the rounding.
    const int g_first = (int)(((blockIdx.x / (unsigned)args_n) * 5u) % (unsigned)n_gran); // by item: every slot of a launch, and a launch of any number of slots, adds in the same order
    auto granule = [&](int g) { // position in H of the share's g-th granule in this workgroup's order
        const int k = min(g, n_gran - 1) + g_first;
        return it.c0 + (k < n_gran ? k : k - n_gran);
    };
    auto load = [&](int g, Regs &r) { // g-th granule of the share, bytes clamped into the row
        const int gg = granule(g);
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int64_t off = min((int64_t)gg * kMsGranuleBytes + h * kMsRowBytes + cb, row_bytes - 16);
#pragma unroll
            for (int i = 0; i < kLoads; ++i) {
                // x rows are read once: streaming loads; page rows come back for the adapter's other
                // token tiles and stay cacheable (measured on 8192-token batches of rank 8 / 128:
                // all plain 77 / 115 us, all streaming 68 / 121 us)
                if (i < MB)
                    r.w[h][i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src[i] + off));
                else
                    r.w[h][i] = *reinterpret_cast<const u32x4 *>(src[i] + off);
            }
        }
    };
    const int last_gran = (int)((row_bytes - 1) / kMsGranuleBytes);
    const bool ragged = row_bytes % kMsGranuleBytes != 0; // only then can a granule reach past the row
    auto stash = [&](int g, int h, const Regs &r) { // half h of granule g -> LDS buffer h; bytes past the row become zero
        unsigned char *buf = lds + h * (kRows * kMsLdsRow);
        const int gg = granule(g);
        if (ragged && gg == last_gran) { // uniform over the workgroup
            const bool ok = (int64_t)gg * kMsGranuleBytes + h * kMsRowBytes + cb < row_bytes;
            const u32x4 zero = u32x4{0u, 0u, 0u, 0u};
#pragma unroll
            for (int i = 0; i < kLoads; ++i)
                *reinterpret_cast<u32x4 *>(buf + (r8 + kMsRowsPerPass * i) * kMsLdsRow + cb) = ok ? r.w[h][i] : zero;
        } else {
#pragma unroll
            for (int i = 0; i < kLoads; ++i)
                *reinterpret_cast<u32x4 *>(buf + (r8 + kMsRowsPerPass * i) * kMsLdsRow + cb) = r.w[h][i];
        }
    };
    // A single rank block would make every MFMA wait for the one before it (they share the
    // accumulator): such tiles keep two accumulators, for alternate k-steps, added at the end.
    constexpr int KA = NB == 1 ? 2 : 1;
    f32x16 acc[NB][KA];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int a = 0; a < KA; ++a)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[nb][a][e] = 0.f;
    auto compute = [&](int h) { // the four k-steps of the chunk in LDS buffer h, for this wavefront's token block
        if (wave >= MB) return;
        const unsigned char *buf = lds + h * (kRows * kMsLdsRow);
#pragma unroll
        for (int k = 0; k < kMsChunk / 16; ++k) {
            const int kb = k * 32 + q * 16; // byte offset of this lane's 8 k-values in the row
            const u32x4 xa = *reinterpret_cast<const u32x4 *>(buf + (wave * 32 + row) * kMsLdsRow + kb);
            u32x4 pb[NB];
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
                pb[nb] = *reinterpret_cast<const u32x4 *>(buf + (32 * MB + nb * 32 + row) * kMsLdsRow + kb);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) acc[nb][k % KA] = mfma32<DT>(xa, pb[nb], acc[nb][k % KA]);
        }
    };

    // register ring: granule g is copied to LDS, half by half, while granule g+1 is still in
    // flight and granule g+2 is requested.  The two halves use the two LDS buffers, one barrier
    // each.  The last granules, which have nothing left to request, are peeled off the loop: its
    // body then has no condition in it, and nothing is fetched that is not used.
    static_assert(kRing == 2, "the peeled loop below is written for a ring of two");
    auto step = [&](int g, Regs &r, bool more) { // `more`: granule g + 2 exists and is requested into r
        stash(g, 0, r);
        __syncthreads();
        compute(0);
        stash(g, 1, r);
        if (more) load(g + 2, r);
        __syncthreads();
        compute(1);
    };
    Regs ring[kRing];
    load(0, ring[0]);
    // keep the granules' loads in issue order: the wait before a granule is copied to LDS then
    // counts only the loads of the younger one as outstanding
    __builtin_amdgcn_sched_barrier(0);
    load(n_gran > 1 ? 1 : 0, ring[1]); // a share of one granule fetches it twice
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (kLoads <= 6) {
        int g = 0;
        for (; g + 3 < n_gran; g += 2) {
            step(g, ring[0], true);
            step(g + 1, ring[1], true);
        }
        // one to three granules are left; only the first of three still has one to request
        step(g, ring[0], g + 2 < n_gran);
        if (g + 1 < n_gran) step(g + 1, ring[1], false);
        if (g + 2 < n_gran) step(g + 2, ring[0], false);
    } else {
        // the widest tiles have no register to spare for the peeled copies: their loop keeps
        // requesting (the last granule again, dropped) to its end
        for (int g = 0; g < n_gran; g += 2) {
            step(g, ring[0], true);
            if (g + 1 < n_gran) step(g + 1, ring[1], true);
        }
    }
    __syncthreads(); // the chunk buffers are free: each wavefront now stages its tiles in its own part

    // ---- accumulator layout -> 8 consecutive ranks of one token per lane -------------------
    // lane l ends up with token l % 32 of its wavefront's v tile and, per 32-rank block, the rank
    // octets l / 32 and l / 32 + 2: exactly the 16 bytes it owns in two operand fragments.
    const int mb_act = (it.ntok + 31) >> 5;          // token blocks / rank blocks that exist
    const int nb_act = (it.nj + 31) >> 5;
    const bool live = wave < mb_act;
    float *stage = reinterpret_cast<float *>(lds) + wave * 32 * kEpiStride;
    float val[NB][2][8];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        if (live && nb < nb_act) {
#pragma unroll
            for (int vv = 0; vv < 16; ++vv) {
                float sum = acc[nb][0][vv];
                if constexpr (KA == 2) sum += acc[nb][1][vv];
                stage[mfma_row(vv, lane) * kEpiStride + row] = sum;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int oct = q + 2 * i;
                const f32x4 lo = *reinterpret_cast<const f32x4 *>(stage + row * kEpiStride + oct * 8);
                const f32x4 hi = *reinterpret_cast<const f32x4 *>(stage + row * kEpiStride + oct * 8 + 4);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    val[nb][i][e] = lo[e];
                    val[nb][i][4 + e] = hi[e];
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
    }

    // ---- a share of a split tile: leave the partial sums for join_shares_kernel ----------------
    if (it.n_parts > 1) {
        if (live) store_share<NB>(it, wave, lane, val, partial);
        return;
    }
    if (live) finish_tile<DT, NB>(it, wave, lane, val, v_stride, vfrag, vexp);
}

template <int DT>
__global__ __launch_bounds__(kMfmaThreads, 2) void shrink_mfma_kernel(const MsItem *__restrict__ items,
                                                                       const int32_t *__restrict__ arena,
                                                                       const uint16_t *__restrict__ pool,
                                                                       const int32_t *__restrict__ tok_idx, int H,
                                                                       int v_stride, MultiArgs args)
{
    // two chunk buffers of (128 token rows + the plan's widest rank block) padded rows, sized at
    // launch: a batch of low-rank adapters leaves room for more workgroups per compute unit
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    // slots vary fastest: the shares of a tile, and the tiles of an adapter, follow one another
    const int cs = blockIdx.x % args.n;
    const MsItem it = items[blockIdx.x / args.n];
    const unsigned char *x = static_cast<const unsigned char *>(args.x[cs]);
    const int32_t *pa = arena + it.arena_off + (int64_t)args.slot[cs] * 2 * it.rank + it.j0;
    uint16_t *vfrag = reinterpret_cast<uint16_t *>(args.v[cs] + args.vfrag_off);
    int8_t *vexp = reinterpret_cast<int8_t *>(args.v[cs] + args.vexp_off);
    float *partial = args.v[cs] + args.part_off + it.part_off;
#define SLORA_MS(NBV, MBV) shrink_mfma_tile<DT, NBV, MBV>(it, pa, x, pool, tok_idx, H, v_stride, vfrag, vexp, partial, lds, args.n)
    if (it.ntok <= 64) {
        if (it.nj <= 32) SLORA_MS(1, 2);
        else if (it.nj <= 64) SLORA_MS(2, 2);
        else SLORA_MS(4, 2);
    } else {
        if (it.nj <= 32) SLORA_MS(1, 4);
        else if (it.nj <= 64) SLORA_MS(2, 4);
        else SLORA_MS(4, 4);
    }
#undef SLORA_MS
}

// One workgroup per split tile, token block and slot; its wavefront nb adds up the shares of rank
// block nb in the order of their numbers (a fixed order: the same bits on every run; the loads of
// four shares are in flight at a time) and finishes the block as the shrink itself does for a
// tile that was not split.  Binary16: the row maximum over the rank blocks meets in LDS.
template <int DT>
__global__ __launch_bounds__(kMfmaThreads) void join_shares_kernel(const MsItem *__restrict__ tiles, int v_stride,
                                                                    MultiArgs args)
{
    constexpr int kBlocks = kMsTok / 32;
    __shared__ float smax[kMsRanks / 32][32];
    const int cs = blockIdx.x % args.n;
    const int tb = (blockIdx.x / args.n) % kBlocks;          // token block
    const MsItem it = tiles[blockIdx.x / args.n / kBlocks];
    const int lane = threadIdx.x & (kWave - 1);
    const int nb = threadIdx.x / kWave;                       // rank block of this wavefront
    const int row = lane & 31, q = lane >> 5;
    const int mb_act = (it.ntok + 31) >> 5, nb_act = (it.nj + 31) >> 5;
    if (tb >= mb_act) return;                                 // the whole workgroup
    const bool live = nb < nb_act;
    float val[2][8];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) val[i][e] = 0.f;
    if (live) {
        const int64_t blk = (int64_t)mb_act * nb_act * 1024;
        const float *base = args.v[cs] + args.part_off + it.part_off + (int64_t)(tb * nb_act + nb) * 1024 + lane * 8;
        constexpr int kBatch = 4;
        for (int p0 = 0; p0 < it.n_parts; p0 += kBatch) {
            f32x4 w[kBatch][4];
#pragma unroll
            for (int k = 0; k < kBatch; ++k) {
                const float *srcp = base + (int64_t)min(p0 + k, it.n_parts - 1) * blk;
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    w[k][2 * i] = *reinterpret_cast<const f32x4 *>(srcp + i * 512);
                    w[k][2 * i + 1] = *reinterpret_cast<const f32x4 *>(srcp + i * 512 + 4);
                }
            }
#pragma unroll
            for (int k = 0; k < kBatch; ++k) {
                if (p0 + k < it.n_parts) {
#pragma unroll
                    for (int i = 0; i < 2; ++i)
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            val[i][e] += w[k][2 * i][e];
                            val[i][4 + e] += w[k][2 * i + 1][e];
                        }
                }
            }
        }
    }
    float sc = 1.f;
    const bool token_ok = tb * 32 + row < it.ntok;
    float vmax = live ? mask_block(it, nb, q, val) : 0.f;
    if constexpr (DT == SLORA_F16) {
        vmax = fmaxf(vmax, __shfl_xor(vmax, 32, kWave));
        if (q == 0) smax[nb][row] = vmax;
        __syncthreads();
#pragma unroll
        for (int k = 0; k < kMsRanks / 32; ++k) vmax = fmaxf(vmax, smax[k][row]);
        const int e = row_exponent(vmax);
        sc = pow2f(e);
        if (nb == 0 && q == 0)
            *vexp_row(reinterpret_cast<int8_t *>(args.v[cs] + args.vexp_off), it, it.tile + tb, v_stride, row) = (int8_t)(token_ok ? e : 0);
    }
    if (live && token_ok)
        store_block<DT>(it, it.tile + tb, nb, lane, val, sc, v_stride,
                        reinterpret_cast<uint16_t *>(args.v[cs] + args.vfrag_off));
}

// ---------------------------------------------------------------------------------------
// prefill expand: y[tok, d] += sum_j V[pos, j] * Bpage_j[d] for a tile of up to 32 tokens and
// up to 256 columns.  The four wavefronts of a workgroup are independent: wavefront w owns
// columns 64w .. 64w+63 (two 32-column MFMA blocks) and keeps a 32 x 64 fp32 tile of y in its
// accumulators - y is loaded INTO the accumulators, the MFMAs add onto it, and it is stored
// once, 128 contiguous bytes per token row and instruction.  Many small independent tiles
// (up to 20 wavefronts per CU) rather than deep software pipelines hide the memory latency.
//
// The first operand is V (tokens x ranks, fp32 in memory).  So that no precision is lost to
// the 16-bit operand format it is split into 16-bit pieces whose sum is V: hi + lo for
// binary16 (22+ bits), hi + mid + lo by truncation for bfloat16 (exactly 24 bits); each piece
// costs one more MFMA on a path that is bound by memory, not by the matrix cores.
// The second operand needs, per lane, 8 consecutive ranks of ONE column, but a page is
// contiguous along columns; the wavefront therefore copies a 32-rank x 64-column slab of B
// through LDS, transposing on the way in (two ranks packed per dword), and reads its operand
// back with one 16-byte LDS load.  Each wavefront uses only its own LDS slab, so the
// workgroup needs no barrier.  All global loads are unconditional: token rows beyond the
// tile, columns beyond the item and ranks beyond the adapter's are redirected to a valid
// row / column / page; what they produce is multiplied by the zero padding of V or is never
// stored.
// ---------------------------------------------------------------------------------------
constexpr int kSlabStride = 20; // dwords per column in LDS: 16 (32 ranks) + 4 pad, keeps 16-byte alignment
constexpr int kSlabGroupPad = 8; // extra dwords before every 8 columns: the 8 column groups a transposing store
                                 // touches then fall into different banks (8 x 20 dwords alone is a multiple of 32:
                                 // rocprofv3 counted bank conflicts on 58 % of this kernel's LDS cycles)
__device__ __forceinline__ int slab_col(int c) { return c * kSlabStride + (c >> 3) * kSlabGroupPad; }
// The y tile of a wavefront (32 rows x 64 columns) is staged in the same slab; padded rows keep the
// 16-byte alignment and spread the accumulator-layout accesses over the banks.
template <bool Y16>
struct YTile;
template <>
struct YTile<true> {
    using type = uint16_t;
    static constexpr int stride = 72;                  // 144-byte rows
    static constexpr int bytes = 32 * stride * 2;
};
template <>
struct YTile<false> {
    using type = float;
    static constexpr int stride = 68;                  // 272-byte rows
    static constexpr int bytes = 32 * stride * 4;
};
constexpr int kSlabBytes = (64 * kSlabStride + 8 * kSlabGroupPad) * 4;

template <int DT, bool Y16>
__global__ __launch_bounds__(kMfmaThreads, 4) void expand_mfma_kernel(const Item *__restrict__ items,
                                                                    const int32_t *__restrict__ arena,
                                                                    const uint16_t *__restrict__ pool,
                                                                    const int32_t *__restrict__ tok_idx, int H,
                                                                    int v_stride, MultiArgs args)
{
    constexpr int kWaveLds = YTile<Y16>::bytes > kSlabBytes ? YTile<Y16>::bytes : kSlabBytes;
    __shared__ u32x4 slab_mem[4][kWaveLds / 16];
    const int cs = mfma_slot_of(blockIdx.x, args.n);
    const Item it = items[mfma_item_of(blockIdx.x, args.n)];
    if (it.ntok == 0) return; // padding of a short per-XCD list
    void *args_y = args.y[cs];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int n = lane & 31;
    const int q = lane >> 5;
    const int col_end = it.a + it.b;        // <= H, multiple of 8
    const int colw = it.a + wave * 64;      // this wavefront's first column
    if (colw >= col_end) return;            // whole wavefront; no barrier is used below
    uint32_t *slab = reinterpret_cast<uint32_t *>(slab_mem[wave]);
    const int32_t *pbl = arena + it.arena_off + (int64_t)args.slot[cs] * 2 * it.rank + it.rank;
    constexpr int NP = VPieces<DT>::N;
    const int n_kk = v_stride >> 4;
    const u32x4 *vfrag = reinterpret_cast<const u32x4 *>(args.v[cs] + args.vfrag_off) + lane;

    const int cg = lane & 7;   // column group (8 columns) this lane copies
    const int kp = lane >> 3;  // rank pair this lane copies
    const int col8 = min(colw + 8 * cg, col_end - 8);
    // page numbers of the four B rows this lane copies per stage, fetched one stage ahead
    int pg[4];
    auto load_pg = [&](int k0) {
#pragma unroll
        for (int rd = 0; rd < 2; ++rd) {
            const int ka = k0 + 16 * rd + 2 * kp;
            pg[2 * rd] = pbl[min(ka, it.rank - 1)];
            pg[2 * rd + 1] = pbl[min(ka + 1, it.rank - 1)];
        }
    };
    load_pg(0);
    // row exponents of the tile's first rank block (binary16 pools), see below
    typedef int32_t e_i32x4 __attribute__((ext_vector_type(4)));
    [[maybe_unused]] const e_i32x4 *vexp_t = nullptr;
    [[maybe_unused]] e_i32x4 e_cur = e_i32x4{0, 0, 0, 0};
    if constexpr (DT == SLORA_F16) {
        const int n_rb = (v_stride + kMsRanks - 1) / kMsRanks;
        vexp_t = reinterpret_cast<const e_i32x4 *>(reinterpret_cast<const int8_t *>(args.v[cs] + args.vexp_off) +
                                                   (int64_t)it.tile * n_rb * 32 + q * 16);
        e_cur = vexp_t[0];
    }

    // accumulators start as the y tile (rows / columns outside the tile read a valid element)
    f32x16 acc[2];
    // The 32 x 64 tile of y passes through the wavefront's LDS slab, which is idle before the
    // first and after the last stage: 16-byte accesses of whole row pieces (128 or 256 bytes)
    // towards memory, single-element LDS accesses in accumulator layout on the other side.
    // A lane moves the kYVec columns of group lane % kYLanes of rows lane / kYLanes + kYRows * i.
    using YT = typename YTile<Y16>::type;
    constexpr int kYVec = 16 / (int)sizeof(YT);   // elements per 16-byte access
    constexpr int kYLanes = 64 / kYVec;           // lanes per tile row
    constexpr int kYRows = kWave / kYLanes;       // rows per access of the wavefront
    constexpr int kYStride = YTile<Y16>::stride;  // padded row, elements
    YT *ytile = reinterpret_cast<YT *>(slab);
    YT *yg = static_cast<YT *>(args_y);
    const int ygrp = lane % kYLanes;
    {
        const int ycol = min(colw + kYVec * ygrp, col_end - kYVec);
#pragma unroll
        for (int i = 0; i < 32 / kYRows; ++i) {
            const int r = lane / kYLanes + kYRows * i;
            const int64_t row = (int64_t)tok_idx[it.pos0 + min(r, it.ntok - 1)] * H;
            const u32x4 w8 = *reinterpret_cast<const u32x4 *>(yg + row + ycol);
            *reinterpret_cast<u32x4 *>(ytile + r * kYStride + kYVec * ygrp) = w8;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int vv = 0; vv < 16; ++vv)
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) {
                const YT e = ytile[mfma_row(vv, lane) * kYStride + nb * 32 + n];
                if constexpr (Y16)
                    acc[nb][vv] = widen1<DT>(e);
                else
                    acc[nb][vv] = e;
            }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront"); // the stages overwrite the slab
    }
    // binary16 pools: the shrink scaled token row i of rank block rb (kMsRanks ranks) by 2^e[rb][i].
    // The accumulators follow: they hold (y + products so far) * 2^e of the CURRENT rank block -
    // scaled up before the first block, re-scaled where the block changes, scaled back at the end.
    // Powers of two: every step is exact.  A lane's 16 exponents of a block are one 16-byte load,
    // requested with the first page numbers (e_cur) so that it has arrived when y has.
    typedef int32_t i32x4 __attribute__((ext_vector_type(4)));
    [[maybe_unused]] auto scale_rows = [&](const i32x4 &from, const i32x4 &to) { // acc *= 2^(to - from), row by row
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int d = (int)(int8_t)(to[g] >> (8 * k)) - (int)(int8_t)(from[g] >> (8 * k));
                const float f = pow2f(d);
                acc[0][4 * g + k] *= f;
                acc[1][4 * g + k] *= f;
            }
    };
    [[maybe_unused]] const i32x4 e_zero = i32x4{0, 0, 0, 0};
    if constexpr (DT == SLORA_F16) scale_rows(e_zero, e_cur);

    for (int k0 = 0; k0 < it.rank; k0 += 32) {
        if constexpr (DT == SLORA_F16) {
            if (k0 > 0 && (k0 & (kMsRanks - 1)) == 0) {
                const i32x4 e_next = vexp_t[(k0 / kMsRanks) * 2];
                scale_rows(e_cur, e_next);
                e_cur = e_next;
            }
        }
        // ---- operands of this stage: two B rows per lane and round, V for both k-steps
        u32x4 wa[2], wb[2];
#pragma unroll
        for (int rd = 0; rd < 2; ++rd) {
            wa[rd] = *reinterpret_cast<const u32x4 *>(pool + (int64_t)pg[2 * rd] * H + col8);
            wb[rd] = *reinterpret_cast<const u32x4 *>(pool + (int64_t)pg[2 * rd + 1] * H + col8);
        }
        load_pg(k0 + 32); // clamped to the last rank past the end
        u32x4 piece[2][NP];
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int p = 0; p < NP; ++p)
                piece[s][p] = vfrag[vfrag_index(it.tile, (k0 >> 4) + s, p, n_kk, NP) / 8];
        // ---- B slab: ranks k0..k0+31 x this wavefront's 64 columns, transposed into LDS
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int rd = 0; rd < 2; ++rd) {
            uint32_t *dst = slab + slab_col(8 * cg) + 8 * rd + kp; // columns 8 cg .. 8 cg + 7: one group, same pad
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                dst[(2 * e) * kSlabStride] = (wa[rd][e] & 0xffffu) | (wb[rd][e] << 16);
                dst[(2 * e + 1) * kSlabStride] = (wa[rd][e] >> 16) | (wb[rd][e] & 0xffff0000u);
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

#pragma unroll
        for (int s = 0; s < 2; ++s) {
            u32x4 bop[2];
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
                bop[nb] = *reinterpret_cast<const u32x4 *>(slab + slab_col(nb * 32 + n) + 8 * s + 4 * q);
#pragma unroll
            for (int p = 0; p < NP; ++p)
#pragma unroll
                for (int nb = 0; nb < 2; ++nb) acc[nb] = mfma32<DT>(piece[s][p], bop[nb], acc[nb]);
        }
    }

    if constexpr (DT == SLORA_F16) scale_rows(e_cur, e_zero);
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int vv = 0; vv < 16; ++vv)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
            YT &e = ytile[mfma_row(vv, lane) * kYStride + nb * 32 + n];
            if constexpr (Y16)
                e = narrow1<DT>(acc[nb][vv]);
            else
                e = acc[nb][vv];
        }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const int ycol = colw + kYVec * ygrp; // a multiple of kYVec, and col_end one of 8: a group is inside or outside
#pragma unroll
    for (int i = 0; i < 32 / kYRows; ++i) {
        const int r = lane / kYLanes + kYRows * i;
        if (r < it.ntok && ycol < col_end) {
            const int64_t row = (int64_t)tok_idx[it.pos0 + r] * H;
            *reinterpret_cast<u32x4 *>(yg + row + ycol) =
                *reinterpret_cast<const u32x4 *>(ytile + r * kYStride + kYVec * ygrp);
        }
    }
}

// ---------------------------------------------------------------------------------------
// Scratch for callers that cannot allocate: v = x*A of one call goes here instead of into a
// buffer from hipMalloc.  One copy per GPU, held until the process ends; every element the
// expand reads is written by the shrink of the same call, so nothing has to start at zero.
// ---------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[SLORA_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_lock;
void *g_scratch_ptr[kMaxDevices]; // device address of `scratch` on each GPU, 0 = not resolved yet

int32_t check_launch(const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(SLORA_EHIP, "%s: %s", what, hipGetErrorString(e));
    return SLORA_OK;
}

} // namespace

// The device address of the static scratch on `device`, which must be the current device: the
// array's name is only a host-side handle, each GPU has its own copy at its own address.
int32_t static_scratch_address(int device, void **out)
{
    *out = nullptr;
    if (device < 0 || device >= kMaxDevices) return fail(SLORA_EINVAL, "device %d outside [0, %d)", device, kMaxDevices);
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (!g_scratch_ptr[device]) {
        void *ptr = nullptr;
        hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr)
            return fail(SLORA_EHIP, "hipGetSymbolAddress(static scratch): %s", hipGetErrorString(e));
        g_scratch_ptr[device] = ptr;
    }
    *out = g_scratch_ptr[device];
    return SLORA_OK;
}

// ---------------------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------------------
int32_t launch_write_pages(slora_pool *pool, const int32_t *d_idx, int64_t n, const void *d_src, void *stream,
                           int32_t max_groups)
{
    if (n <= 0) return SLORA_OK;
    if (n >= (int64_t(1) << 31)) return fail(SLORA_EINVAL, "too many pages in one call");
    if (reinterpret_cast<uintptr_t>(d_src) & 15) return fail(SLORA_EINVAL, "src must be 16-byte aligned");
    const int64_t groups = max_groups > 0 && n > max_groups ? max_groups : n;
    hipLaunchKernelGGL(write_pages_kernel, dim3((unsigned)groups), dim3(256), 0, (hipStream_t)stream,
                       static_cast<uint16_t *>(pool->dev_base), d_idx, static_cast<const uint16_t *>(d_src), pool->H, n);
    return check_launch("write_pages");
}

int32_t launch_gather(slora_pool *pool, int64_t arena_entry, int32_t rank, void *dev_out, void *stream)
{
    hipLaunchKernelGGL(gather_pages_kernel, dim3((unsigned)rank), dim3(256), 0, (hipStream_t)stream,
                       static_cast<const uint16_t *>(pool->dev_base), pool->d_arena + arena_entry,
                       static_cast<uint16_t *>(dev_out), pool->H);
    return check_launch("gather_pages");
}

// loads per block of the vector shrink: as few blocks per page as 8 loads allow, then the smallest U that fits
static int shrink_loads_per_block(int H)
{
    const int per_lane = (H / 8 + kWave - 1) / kWave;
    const int nblk = (per_lane + 7) / 8;
    return std::max(4, (per_lane + nblk - 1) / nblk);
}

int32_t launch_fused(slora_plan *plan, int32_t n, const MultiArgs &args, void *stream, bool y16)
{
    slora_pool *pool = plan->pool;
    if (plan->vf_items.empty()) return SLORA_OK;
    const uint16_t *base = static_cast<const uint16_t *>(pool->dev_base);
    hipStream_t st = (hipStream_t)stream;
    const int H = pool->H;
    const int strips = (H + 511) / 512;
    const dim3 block((unsigned)(std::min(strips, 16) * kWave));
    const dim3 grid((unsigned)(plan->vf_items.size() * (size_t)n));
    const int v_pad = plan->v_stride;
    const size_t lds = (size_t)kExpandTok * H * 2 + (size_t)kExpandTok * v_pad * sizeof(float);
    const int U = shrink_loads_per_block(H);
    // more than 64 KiB of dynamic LDS (H = 8192) has to be allowed once per kernel instance
    hipError_t attr = hipSuccess;
#define SLORA_FUSED(DT, Y, UU)                                                                                       \
    {                                                                                                                \
        static bool allowed = false;                                                                                 \
        if (!allowed && lds > 65536) {                                                                               \
            attr = hipFuncSetAttribute(reinterpret_cast<const void *>(&lora_vec_fused_kernel<DT, Y, UU>),           \
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);                      \
            allowed = attr == hipSuccess;                                                                            \
        }                                                                                                            \
        if (attr == hipSuccess)                                                                                      \
            hipLaunchKernelGGL((lora_vec_fused_kernel<DT, Y, UU>), grid, block, lds, st, plan->d_vf, pool->d_arena, \
                               base, plan->d_tok_idx, H, v_pad, args);                                               \
    }
#define SLORA_FUSED_U(DT, Y)                      \
    switch (U) {                                  \
    case 4: SLORA_FUSED(DT, Y, 4); break;         \
    case 5: SLORA_FUSED(DT, Y, 5); break;         \
    case 6: SLORA_FUSED(DT, Y, 6); break;         \
    case 7: SLORA_FUSED(DT, Y, 7); break;         \
    default: SLORA_FUSED(DT, Y, 8); break;        \
    }
    if (pool->dtype == SLORA_F16) {
        if (y16) { SLORA_FUSED_U(SLORA_F16, true) } else { SLORA_FUSED_U(SLORA_F16, false) }
    } else {
        if (y16) { SLORA_FUSED_U(SLORA_BF16, true) } else { SLORA_FUSED_U(SLORA_BF16, false) }
    }
#undef SLORA_FUSED_U
#undef SLORA_FUSED
    if (attr != hipSuccess) return fail(SLORA_EHIP, "hipFuncSetAttribute(LDS size): %s", hipGetErrorString(attr));
    return check_launch("lora_vec_fused");
}

int32_t launch_shrink(slora_plan *plan, int32_t n, const MultiArgs &args, void *stream, bool heads_only)
{
    slora_pool *pool = plan->pool;
    const uint16_t *base = static_cast<const uint16_t *>(pool->dev_base);
    hipStream_t st = (hipStream_t)stream;
    const size_t n_vs = heads_only ? (size_t)plan->n_vs_head : plan->vs_items.size();
    if (n_vs > 0) {
        const dim3 grid((unsigned)(n_vs * (size_t)n));
        const size_t lds = (size_t)plan->max_shrink_tok * pool->H * 2;
        const int U = shrink_loads_per_block(pool->H);
#define SLORA_LAUNCH_SHRINK(DT, UU)                                                                              \
    hipLaunchKernelGGL((shrink_vec_kernel<DT, UU>), grid, dim3(kShrinkThreads), lds, st, plan->d_vs, pool->d_arena, \
                       base, plan->d_tok_idx, pool->H, plan->v_stride, args)
#define SLORA_SHRINK_U(DT)                                \
    switch (U) {                                          \
    case 4: SLORA_LAUNCH_SHRINK(DT, 4); break;            \
    case 5: SLORA_LAUNCH_SHRINK(DT, 5); break;            \
    case 6: SLORA_LAUNCH_SHRINK(DT, 6); break;            \
    case 7: SLORA_LAUNCH_SHRINK(DT, 7); break;            \
    default: SLORA_LAUNCH_SHRINK(DT, 8); break;           \
    }
        if (pool->dtype == SLORA_F16) {
            SLORA_SHRINK_U(SLORA_F16)
        } else {
            SLORA_SHRINK_U(SLORA_BF16)
        }
#undef SLORA_SHRINK_U
#undef SLORA_LAUNCH_SHRINK
        int32_t rc = check_launch("shrink_vec");
        if (rc != SLORA_OK) return rc;
    }
    if (!plan->ms_items.empty()) {
        const dim3 grid((unsigned)(plan->ms_items.size() * (size_t)n));
        // LDS: the kernel's two chunk buffers for the widest tile of this plan (never less than the
        // four staging tiles of the epilogue)
        const int nb_max = plan->ms_max_nj <= 32 ? 1 : plan->ms_max_nj <= 64 ? 2 : 4;
        const size_t lds = std::max<size_t>((size_t)2 * (kMsTok + 32 * nb_max) * kMsLdsRow, (size_t)4 * 32 * kEpiStride * sizeof(float));
        if (pool->dtype == SLORA_F16)
            hipLaunchKernelGGL(shrink_mfma_kernel<SLORA_F16>, grid, dim3(kMfmaThreads), lds, st, plan->d_ms,
                               pool->d_arena, base, plan->d_tok_idx, pool->H, plan->v_stride, args);
        else
            hipLaunchKernelGGL(shrink_mfma_kernel<SLORA_BF16>, grid, dim3(kMfmaThreads), lds, st, plan->d_ms,
                               pool->d_arena, base, plan->d_tok_idx, pool->H, plan->v_stride, args);
        int32_t rc = check_launch("shrink_mfma");
        if (rc != SLORA_OK) return rc;
        if (plan->n_sync > 0) {
            const dim3 jgrid((unsigned)((size_t)plan->n_sync * (kMsTok / 32) * (size_t)n));
            if (pool->dtype == SLORA_F16)
                hipLaunchKernelGGL(join_shares_kernel<SLORA_F16>, jgrid, dim3(kMfmaThreads), 0, st, plan->d_mj,
                                   plan->v_stride, args);
            else
                hipLaunchKernelGGL(join_shares_kernel<SLORA_BF16>, jgrid, dim3(kMfmaThreads), 0, st, plan->d_mj,
                                   plan->v_stride, args);
            rc = check_launch("join_shares");
            if (rc != SLORA_OK) return rc;
        }
    }
    return SLORA_OK;
}

int32_t launch_expand(slora_plan *plan, int32_t n, const MultiArgs &args, void *stream, bool y16, bool heads_only)
{
    slora_pool *pool = plan->pool;
    const uint16_t *base = static_cast<const uint16_t *>(pool->dev_base);
    hipStream_t st = (hipStream_t)stream;
    // (storage type, y type) -> kernel instance
#define SLORA_PICK(KERNEL)                                                                   \
    (pool->dtype == SLORA_F16 ? (y16 ? KERNEL<SLORA_F16, true> : KERNEL<SLORA_F16, false>)   \
                              : (y16 ? KERNEL<SLORA_BF16, true> : KERNEL<SLORA_BF16, false>))
    const size_t n_ve = heads_only ? (size_t)plan->n_ve_head : plan->ve_items.size();
    if (n_ve > 0) {
        const dim3 grid((unsigned)(n_ve * (size_t)n));
        if (plan->expand_split)
            hipLaunchKernelGGL(SLORA_PICK(expand_vec_split_kernel), grid, dim3(kSplitWaves * kWave), 0, st, plan->d_ve,
                               pool->d_arena, base, plan->d_tok_idx, pool->H, plan->v_stride, args);
        else
            hipLaunchKernelGGL(SLORA_PICK(expand_vec_kernel), grid, dim3((unsigned)plan->expand_threads), 0, st,
                               plan->d_ve, pool->d_arena, base, plan->d_tok_idx, pool->H, plan->v_stride, args);
        int32_t rc = check_launch("expand_vec");
        if (rc != SLORA_OK) return rc;
    }
    if (!plan->me_items.empty()) {
        const dim3 grid((unsigned)(plan->me_items.size() * (size_t)n));
        hipLaunchKernelGGL(SLORA_PICK(expand_mfma_kernel), grid, dim3(kMfmaThreads), 0, st, plan->d_me, pool->d_arena,
                           base, plan->d_tok_idx, pool->H, plan->v_stride, args);
        int32_t rc = check_launch("expand_mfma");
        if (rc != SLORA_OK) return rc;
    }
#undef SLORA_PICK
    return SLORA_OK;
}

} // namespace slora
