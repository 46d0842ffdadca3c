// gfx950 (CDNA4) kernels: page scatter/gather, and the shrink / expand pair of the batched
// LoRA term (Sec. 5.3: gather matrix-vector for decode, gather matrix-matrix for prefill).
//
// Data layout: pool = n_pages rows of H 16-bit elements; an adapter's page lists sit in an
// int32 arena as [slot][A columns r][B rows r]; x is T x H (16-bit), y is T x H (fp32),
// v = x*A is kept in fp32 as rows of `v_stride` floats indexed by the token's position in the
// plan's sorted token list.  All byte offsets into the pool are 64-bit.
#include <hip/hip_runtime.h>

#include "slora_internal.hpp"

namespace slora {

namespace {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

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
                                                           const uint16_t *__restrict__ src, int H)
{
    const int64_t i = blockIdx.x;
    const u32x4 *s = reinterpret_cast<const u32x4 *>(src + i * H);
    u32x4 *d = reinterpret_cast<u32x4 *>(pool + (int64_t)idx[i] * H);
    for (int c = threadIdx.x; c < H / 8; c += blockDim.x) d[c] = s[c];
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
// One workgroup (4 wavefronts) = one item = up to kShrinkPages pages of one adapter and up to
// kShrinkTok tokens that use it.  The tokens' x rows are staged once in LDS; each wavefront
// then streams whole pages from HBM with 16-byte loads per lane (8 in flight), dots them
// against the staged rows with packed 16-bit dot products accumulating in fp32, and reduces
// across the 64 lanes.
// ---------------------------------------------------------------------------------------
constexpr int kShrinkThreads = 256;
constexpr int kShrinkUnroll = 8;

template <int DT>
__global__ __launch_bounds__(kShrinkThreads) void shrink_vec_kernel(const Item *__restrict__ items,
                                                                     const int32_t *__restrict__ arena,
                                                                     const uint16_t *__restrict__ pool,
                                                                     const int32_t *__restrict__ tok_idx, int H,
                                                                     int v_stride, MultiArgs args)
{
    extern __shared__ u32x4 xs[]; // [ntok][H/8]
    const Item it = items[blockIdx.x];
    const int cs = blockIdx.y;
    const uint16_t *__restrict__ x = static_cast<const uint16_t *>(args.x[cs]);
    float *__restrict__ v = args.v[cs];
    const int nch = H >> 3; // 16-byte chunks per row
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;

    for (int t = 0; t < it.ntok; ++t) {
        const u32x4 *row = reinterpret_cast<const u32x4 *>(x + (int64_t)tok_idx[it.pos0 + t] * H);
        for (int c = tid; c < nch; c += kShrinkThreads) xs[t * nch + c] = row[c];
    }
    __syncthreads();

    const int32_t *pa = arena + it.arena_off + (int64_t)args.slot[cs] * 2 * it.rank;
    const u32x4 zero = u32x4{0u, 0u, 0u, 0u};
    for (int jj = wave; jj < it.b; jj += kShrinkThreads / kWave) {
        const int j = it.a + jj;
        const u32x4 *page = reinterpret_cast<const u32x4 *>(pool + (int64_t)pa[j] * H);
        float acc[kShrinkTok];
#pragma unroll
        for (int t = 0; t < kShrinkTok; ++t) acc[t] = 0.f;
        for (int c0 = 0; c0 < nch; c0 += kWave * kShrinkUnroll) {
            u32x4 w[kShrinkUnroll];
#pragma unroll
            for (int u = 0; u < kShrinkUnroll; ++u) {
                const int c = c0 + u * kWave + lane;
                w[u] = c < nch ? __builtin_nontemporal_load(page + c) : zero;
            }
#pragma unroll
            for (int t = 0; t < kShrinkTok; ++t) {
                if (t < it.ntok) {
#pragma unroll
                    for (int u = 0; u < kShrinkUnroll; ++u) {
                        const int c = c0 + u * kWave + lane;
                        const u32x4 xv = c < nch ? xs[t * nch + c] : zero;
                        acc[t] = dot8<DT>(w[u], xv, acc[t]);
                    }
                }
            }
        }
#pragma unroll
        for (int t = 0; t < kShrinkTok; ++t) {
            if (t < it.ntok) {
                const float s = wave_sum(acc[t]);
                if (lane == 0) v[(int64_t)(it.pos0 + t) * v_stride + j] = s;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// decode path, expand: y[tok, d] += sum_j v[pos, j] * Bpage_j[d]
//
// One wavefront = one item = 512 columns of one adapter's B for up to kExpandTok tokens.  Each
// lane owns 8 adjacent columns: it streams 16 bytes of every B row (8 rows in flight), widens
// to fp32 and accumulates v[pos, j] * row for every token, then does one read-modify-write of
// its 8 floats of y per token (a wavefront covers 2 KiB of a y row).
// ---------------------------------------------------------------------------------------
constexpr int kExpandUnroll = 8;

template <int DT>
__global__ __launch_bounds__(kWave) void expand_vec_kernel(const Item *__restrict__ items,
                                                            const int32_t *__restrict__ arena,
                                                            const uint16_t *__restrict__ pool,
                                                            const int32_t *__restrict__ tok_idx, int H, int v_stride,
                                                            MultiArgs args)
{
    const Item it = items[blockIdx.x];
    const int cs = blockIdx.y;
    float *__restrict__ y = args.y[cs];
    const float *__restrict__ v = args.v[cs];
    const int lane = threadIdx.x;
    const int col = it.a + lane * 8;
    const bool live = col < H;
    const int32_t *pb = arena + it.arena_off + (int64_t)args.slot[cs] * 2 * it.rank + it.rank;
    const float *vrow = v + (int64_t)it.pos0 * v_stride;

    float acc[kExpandTok][8];
#pragma unroll
    for (int t = 0; t < kExpandTok; ++t)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[t][e] = 0.f;

    const u32x4 zero = u32x4{0u, 0u, 0u, 0u};
    for (int j0 = 0; j0 < it.rank; j0 += kExpandUnroll) {
        u32x4 w[kExpandUnroll];
#pragma unroll
        for (int u = 0; u < kExpandUnroll; ++u) {
            const int j = j0 + u;
            w[u] = (j < it.rank && live)
                       ? __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(pool + (int64_t)pb[j] * H + col))
                       : zero;
        }
#pragma unroll
        for (int u = 0; u < kExpandUnroll; ++u) {
            const int j = j0 + u;
            if (j < it.rank) {
                float f[8];
                widen2<DT>(w[u].x, f[0], f[1]);
                widen2<DT>(w[u].y, f[2], f[3]);
                widen2<DT>(w[u].z, f[4], f[5]);
                widen2<DT>(w[u].w, f[6], f[7]);
#pragma unroll
                for (int t = 0; t < kExpandTok; ++t) {
                    if (t < it.ntok) {
                        const float vv = vrow[t * v_stride + j];
#pragma unroll
                        for (int e = 0; e < 8; ++e) acc[t][e] = fmaf(vv, f[e], acc[t][e]);
                    }
                }
            }
        }
    }
    if (!live) return;
#pragma unroll
    for (int t = 0; t < kExpandTok; ++t) {
        if (t < it.ntok) {
            float4 *yp = reinterpret_cast<float4 *>(y + (int64_t)tok_idx[it.pos0 + t] * H + col);
            float4 a = yp[0], b = yp[1];
            a.x += acc[t][0];
            a.y += acc[t][1];
            a.z += acc[t][2];
            a.w += acc[t][3];
            b.x += acc[t][4];
            b.y += acc[t][5];
            b.z += acc[t][6];
            b.w += acc[t][7];
            yp[0] = a;
            yp[1] = b;
        }
    }
}

int32_t check_launch(const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(SLORA_EHIP, "%s: %s", what, hipGetErrorString(e));
    return SLORA_OK;
}

} // namespace

// ---------------------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------------------
int32_t launch_write_pages(slora_pool *pool, const int32_t *d_idx, int64_t n, const void *d_src, void *stream)
{
    if (n <= 0) return SLORA_OK;
    if (n >= (int64_t(1) << 31)) return fail(SLORA_EINVAL, "too many pages in one call");
    if (reinterpret_cast<uintptr_t>(d_src) & 15) return fail(SLORA_EINVAL, "src must be 16-byte aligned");
    hipLaunchKernelGGL(write_pages_kernel, dim3((unsigned)n), dim3(256), 0, (hipStream_t)stream,
                       static_cast<uint16_t *>(pool->dev_base), d_idx, static_cast<const uint16_t *>(d_src), pool->H);
    return check_launch("write_pages");
}

int32_t launch_gather(slora_pool *pool, int64_t arena_entry, int32_t rank, void *dev_out, void *stream)
{
    hipLaunchKernelGGL(gather_pages_kernel, dim3((unsigned)rank), dim3(256), 0, (hipStream_t)stream,
                       static_cast<const uint16_t *>(pool->dev_base), pool->d_arena + arena_entry,
                       static_cast<uint16_t *>(dev_out), pool->H);
    return check_launch("gather_pages");
}

int32_t launch_shrink(slora_plan *plan, int32_t n, const MultiArgs &args, void *stream)
{
    slora_pool *pool = plan->pool;
    const uint16_t *base = static_cast<const uint16_t *>(pool->dev_base);
    hipStream_t st = (hipStream_t)stream;
    if (!plan->ms_items.empty()) return fail(SLORA_EINVAL, "MFMA path is not available in this build");
    if (!plan->vs_items.empty()) {
        const dim3 grid((unsigned)plan->vs_items.size(), (unsigned)n);
        const size_t lds = (size_t)plan->max_shrink_tok * pool->H * 2;
        if (pool->dtype == SLORA_F16)
            hipLaunchKernelGGL(shrink_vec_kernel<SLORA_F16>, grid, dim3(kShrinkThreads), lds, st, plan->d_vs,
                               pool->d_arena, base, plan->d_tok_idx, pool->H, plan->v_stride, args);
        else
            hipLaunchKernelGGL(shrink_vec_kernel<SLORA_BF16>, grid, dim3(kShrinkThreads), lds, st, plan->d_vs,
                               pool->d_arena, base, plan->d_tok_idx, pool->H, plan->v_stride, args);
        int32_t rc = check_launch("shrink_vec");
        if (rc != SLORA_OK) return rc;
    }
    return SLORA_OK;
}

int32_t launch_expand(slora_plan *plan, int32_t n, const MultiArgs &args, void *stream)
{
    slora_pool *pool = plan->pool;
    const uint16_t *base = static_cast<const uint16_t *>(pool->dev_base);
    hipStream_t st = (hipStream_t)stream;
    if (!plan->me_items.empty()) return fail(SLORA_EINVAL, "MFMA path is not available in this build");
    if (!plan->ve_items.empty()) {
        const dim3 grid((unsigned)plan->ve_items.size(), (unsigned)n);
        if (pool->dtype == SLORA_F16)
            hipLaunchKernelGGL(expand_vec_kernel<SLORA_F16>, grid, dim3(kWave), 0, st, plan->d_ve, pool->d_arena, base,
                               plan->d_tok_idx, pool->H, plan->v_stride, args);
        else
            hipLaunchKernelGGL(expand_vec_kernel<SLORA_BF16>, grid, dim3(kWave), 0, st, plan->d_ve, pool->d_arena, base,
                               plan->d_tok_idx, pool->H, plan->v_stride, args);
        int32_t rc = check_launch("expand_vec");
        if (rc != SLORA_OK) return rc;
    }
    return SLORA_OK;
}

} // namespace slora
