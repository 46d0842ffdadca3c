/*
 * CPU fp64 oracle for heterogeneous batched LoRA over a paged pool.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may call into this file; it exists so
 * that tests, the smoke check and the bench's cpu_baseline leg have a slow, obviously correct
 * answer to compare the GPU kernels against.  It shares no code, header, table or helper with
 * the HIP library.
 *
 * What it computes, per token t with adapter i = ids[t] (paper Sec. 2, Eq. 2, the `xAB` term
 * that Fig. 1's `add` node adds onto the base model's `xW`; one adapter per token as in
 * Sec. 4.1):
 *
 *     v[j]      = sum_h x[t,h] * A_i[h,j]                    j < r_i
 *     y_out[t,d] = y_in[t,d] + sum_j v[j] * B_i[j,d]
 *
 * with A_i and B_i read through page lists (Sec. 5.1: a page is one H-vector; a rank-r LoRA
 * matrix takes r pages, stored non-contiguously).  Page j of the A list holds column j of A,
 * page j of the B list holds row j of B, so both are H-vectors.  There is no alpha/r scaling
 * (Eq. 1-2 carry none).  Tokens with id -1, and adapters of rank 0, leave their row of y
 * untouched.  All arithmetic is fp64 on the exact values of the 16-bit inputs; loops run in
 * the order the definition states, with no blocking or fusion.  OpenMP only distributes
 * tokens, which are independent.
 *
 * Parity pins live in tests/ (dense x(AB) materialisation, padded batched-matmul form,
 * one-hot closed forms, hand-worked examples, invariances); nothing here is unpinned.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { SLO_F16 = 0, SLO_BF16 = 1 };

/* IEEE binary16 -> double, exact (1 sign, 5 exponent bits bias 15, 10 fraction bits). */
double slo_f16_to_f64(uint16_t b)
{
    int sign = (b >> 15) & 1;
    int e = (b >> 10) & 0x1f;
    int f = b & 0x3ff;
    double m;
    if (e == 0)
        m = ldexp((double)f, -24);                 /* zero and subnormals: f * 2^-10 * 2^-14 */
    else if (e == 31)
        m = f ? NAN : INFINITY;
    else
        m = ldexp((double)(f | 0x400), e - 25);    /* (1 + f/1024) * 2^(e-15) */
    return sign ? -m : m;
}

/* bfloat16 -> double, exact (1 sign, 8 exponent bits bias 127, 7 fraction bits). */
double slo_bf16_to_f64(uint16_t b)
{
    int sign = (b >> 15) & 1;
    int e = (b >> 7) & 0xff;
    int f = b & 0x7f;
    double m;
    if (e == 0)
        m = ldexp((double)f, -133);                /* f * 2^-7 * 2^-126 */
    else if (e == 255)
        m = f ? NAN : INFINITY;
    else
        m = ldexp((double)(f | 0x80), e - 134);    /* (1 + f/128) * 2^(e-127) */
    return sign ? -m : m;
}

static double widen(uint16_t b, int dtype)
{
    return dtype == SLO_F16 ? slo_f16_to_f64(b) : slo_bf16_to_f64(b);
}

/* Widen n raw 16-bit patterns (for tests of the two decoders). */
void slo_widen(const uint16_t *bits, int64_t n, int dtype, double *out)
{
    for (int64_t i = 0; i < n; ++i)
        out[i] = widen(bits[i], dtype);
}

/*
 * Gather a paged matrix: out[j*H + h] = pool[pages[j]*H + h], j < r, widened exactly.
 * Returns 0, or -1 if a page index is outside [0, n_pages).
 */
int slo_gather(const uint16_t *pool, int64_t n_pages, int64_t H, int dtype,
               const int32_t *pages, int32_t r, double *out)
{
    for (int32_t j = 0; j < r; ++j) {
        if (pages[j] < 0 || (int64_t)pages[j] >= n_pages)
            return -1;
        const uint16_t *row = pool + (int64_t)pages[j] * H;
        for (int64_t h = 0; h < H; ++h)
            out[(int64_t)j * H + h] = widen(row[h], dtype);
    }
    return 0;
}

/* Same gather, raw bits (what a bit-exact page gather must return). */
int slo_gather_bits(const uint16_t *pool, int64_t n_pages, int64_t H,
                    const int32_t *pages, int32_t r, uint16_t *out)
{
    for (int32_t j = 0; j < r; ++j) {
        if (pages[j] < 0 || (int64_t)pages[j] >= n_pages)
            return -1;
        memcpy(out + (int64_t)j * H, pool + (int64_t)pages[j] * H, (size_t)H * sizeof(uint16_t));
    }
    return 0;
}

/*
 * y_out = y_in + per-token x A_i B_i for ONE slot (one projection of one layer).
 *
 *   pool       n_pages * H raw 16-bit patterns
 *   rank       [n_adapters]
 *   list_off   [n_adapters] offset into page_lists of this slot's 2*rank entries:
 *              first the rank pages of A (columns), then the rank pages of B (rows)
 *   ids        [T] adapter per token, -1 = none
 *   x          [T*H] raw 16-bit patterns, row-major
 *   y_in       [T*H] fp32, y_out [T*H] fp64
 *   n_threads  OpenMP threads over tokens (<=0: runtime default)
 *
 * Returns 0, -1 on a page index out of range, -2 on an adapter id out of range.
 * Returns the number of threads actually used through *threads_used when non-NULL.
 */
int slo_lora_apply(const uint16_t *pool, int64_t n_pages, int32_t H, int dtype,
                   const int32_t *rank, const int64_t *list_off, const int32_t *page_lists,
                   int32_t n_adapters, const int32_t *ids, int32_t T,
                   const uint16_t *x, const float *y_in, double *y_out,
                   int n_threads, int *threads_used)
{
    int err = 0;
    int used = 1;
#ifdef _OPENMP
    if (n_threads <= 0)
        n_threads = omp_get_max_threads();
#else
    n_threads = 1;
#endif
    /* validate before touching anything */
    for (int32_t t = 0; t < T; ++t) {
        int32_t i = ids[t];
        if (i == -1)
            continue;
        if (i < 0 || i >= n_adapters)
            return -2;
        const int32_t *pl = page_lists + list_off[i];
        for (int32_t j = 0; j < 2 * rank[i]; ++j)
            if (pl[j] < 0 || (int64_t)pl[j] >= n_pages)
                return -1;
    }
#pragma omp parallel num_threads(n_threads)
    {
#ifdef _OPENMP
#pragma omp single
        used = omp_get_num_threads();
#endif
        double *v = NULL;
        int32_t v_cap = 0;
#pragma omp for schedule(dynamic, 1)
        for (int32_t t = 0; t < T; ++t) {
            double *yo = y_out + (int64_t)t * H;
            const float *yi = y_in + (int64_t)t * H;
            for (int32_t d = 0; d < H; ++d)
                yo[d] = (double)yi[d];
            int32_t i = ids[t];
            if (i == -1)
                continue;
            int32_t r = rank[i];
            if (r == 0)
                continue;
            if (r > v_cap) {
                free(v);
                v = (double *)malloc((size_t)r * sizeof(double));
                v_cap = r;
                if (!v) {
#pragma omp atomic write
                    err = -3;
                    v_cap = 0;
                    continue;
                }
            }
            const int32_t *pa = page_lists + list_off[i];       /* columns of A */
            const int32_t *pb = pa + r;                         /* rows of B    */
            const uint16_t *xt = x + (int64_t)t * H;
            /* shrink: v = x A */
            for (int32_t j = 0; j < r; ++j) {
                const uint16_t *acol = pool + (int64_t)pa[j] * H;
                double s = 0.0;
                for (int32_t h = 0; h < H; ++h)
                    s += widen(xt[h], dtype) * widen(acol[h], dtype);
                v[j] = s;
            }
            /* expand: y += v B */
            for (int32_t d = 0; d < H; ++d) {
                double s = 0.0;
                for (int32_t j = 0; j < r; ++j)
                    s += v[j] * widen(pool[(int64_t)pb[j] * H + d], dtype);
                yo[d] += s;
            }
        }
        free(v);
    }
    if (threads_used)
        *threads_used = used;
    return err;
}

/*
 * 16-bit output (the variant in which y has the pool's storage type instead of fp32).
 *
 * The definition is unchanged - y_out = y_in + x A_i B_i (Sec. 2, Eq. 2) - and the result is
 * then rounded ONCE, from the fp64 value, to the nearest binary16 / bfloat16 value, ties to
 * even (IEEE 754 roundTiesToEven): gradual underflow to subnormals, overflow to infinity, NaN
 * stays NaN.  A 16-bit y_in is exact in fp32, so the caller widens it and uses slo_lora_apply;
 * this function is only the final rounding.
 */
uint16_t slo_f64_to_16(double v, int dtype)
{
    const int p = dtype == SLO_F16 ? 11 : 8;          /* significand bits, hidden one included */
    const int emin = dtype == SLO_F16 ? -14 : -126;   /* exponent of the smallest normal value */
    const int emax = dtype == SLO_F16 ? 15 : 127;     /* exponent of the largest finite value  */
    const int fbits = p - 1;
    const uint16_t sign = signbit(v) ? 0x8000u : 0u;
    const uint16_t inf = (uint16_t)(((2 * emax + 1) << fbits));   /* exponent field all ones */
    if (isnan(v))
        return (uint16_t)(sign | inf | (1u << (fbits - 1)));
    double a = fabs(v);
    if (isinf(a))
        return (uint16_t)(sign | inf);
    if (a == 0.0)
        return sign;
    int e;
    (void)frexp(a, &e);
    e -= 1;                              /* a = m * 2^e with 1 <= m < 2 */
    if (e < emin)
        e = emin;                        /* subnormal range: the spacing stops shrinking */
    /* a in units of the last place at exponent e; nearbyint rounds ties to even in the default
       rounding mode; the scaling by a power of two is exact */
    double n = nearbyint(ldexp(a, fbits - e));
    if (n >= ldexp(1.0, p)) {            /* rounded up into the next binade */
        n = ldexp(1.0, fbits);
        e += 1;
    }
    if (e > emax)
        return (uint16_t)(sign | inf);
    uint32_t N = (uint32_t)n;
    if (N < (1u << fbits))               /* no hidden one: subnormal (e == emin) or zero */
        return (uint16_t)(sign | N);
    return (uint16_t)(sign | ((uint32_t)(e + emax) << fbits) | (N - (1u << fbits)));
}

void slo_round16(const double *v, int64_t n, int dtype, uint16_t *out)
{
    for (int64_t i = 0; i < n; ++i)
        out[i] = slo_f64_to_16(v[i], dtype);
}
