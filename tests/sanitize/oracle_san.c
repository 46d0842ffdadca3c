/* The C oracle under AddressSanitizer / UndefinedBehaviorSanitizer: every exported function on
 * exact-size heap buffers (so that one element too far is reported), edge cases included
 * (no tokens, tokens without adapter, rank 0, every 16-bit pattern through the decoders and
 * through the rounding, bad indices refused before anything is read).  It checks memory safety
 * and the error codes; the values are pinned by tests/test_oracle_pins.py. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

double slo_f16_to_f64(uint16_t b);
double slo_bf16_to_f64(uint16_t b);
void slo_widen(const uint16_t *bits, int64_t n, int dtype, double *out);
int slo_gather(const uint16_t *pool, int64_t n_pages, int64_t H, int dtype, const int32_t *pages, int32_t r, double *out);
int slo_gather_bits(const uint16_t *pool, int64_t n_pages, int64_t H, const int32_t *pages, int32_t r, uint16_t *out);
int slo_lora_apply(const uint16_t *pool, int64_t n_pages, int32_t H, int dtype, const int32_t *rank,
                   const int64_t *list_off, const int32_t *page_lists, int32_t n_adapters, const int32_t *ids,
                   int32_t T, const uint16_t *x, const float *y_in, double *y_out, int n_threads, int *threads_used);
uint16_t slo_f64_to_16(double v, int dtype);
void slo_round16(const double *v, int64_t n, int dtype, uint16_t *out);

#define REQUIRE(c) do { if (!(c)) { fprintf(stderr, "oracle_san: %s failed at line %d\n", #c, __LINE__); abort(); } } while (0)

static uint32_t state = 12345u;
static uint32_t rnd(void) { state = state * 1664525u + 1013904223u; return state >> 8; }

int main(void)
{
    /* decoders and rounding over all patterns; rounding a decoded value gives the pattern back */
    for (int dtype = 0; dtype < 2; ++dtype) {
        uint16_t *bits = malloc(65536 * sizeof *bits);
        double *val = malloc(65536 * sizeof *val);
        uint16_t *back = malloc(65536 * sizeof *back);
        for (int b = 0; b < 65536; ++b) bits[b] = (uint16_t)b;
        slo_widen(bits, 65536, dtype, val);
        slo_round16(val, 65536, dtype, back);
        for (int b = 0; b < 65536; ++b) {
            REQUIRE(isnan(val[b]) ? (isnan(dtype ? slo_bf16_to_f64(back[b]) : slo_f16_to_f64(back[b]))) : back[b] == bits[b]);
            REQUIRE(isnan(val[b]) || val[b] == (dtype ? slo_bf16_to_f64((uint16_t)b) : slo_f16_to_f64((uint16_t)b)));
        }
        REQUIRE(slo_f64_to_16(1e300, dtype) == (dtype ? 0x7f80 : 0x7c00));
        REQUIRE(slo_f64_to_16(-1e-300, dtype) == 0x8000);
        free(bits); free(val); free(back);
    }
    /* apply on exact-size buffers */
    for (int round = 0; round < 40; ++round) {
        const int32_t H = 8 * (1 + (int32_t)(rnd() % 12)), n_ad = 1 + (int32_t)(rnd() % 5), T = (int32_t)(rnd() % 9);
        const int dtype = (int)(rnd() & 1);
        int32_t *rank = malloc((size_t)n_ad * sizeof *rank);
        int64_t *off = malloc((size_t)n_ad * sizeof *off);
        int64_t total = 0;
        for (int a = 0; a < n_ad; ++a) { rank[a] = (int32_t)(rnd() % 7); off[a] = total; total += 2 * rank[a]; }
        const int64_t n_pages = total + 3;
        int32_t *lists = malloc((size_t)(total ? total : 1) * sizeof *lists);
        for (int64_t k = 0; k < total; ++k) lists[k] = (int32_t)((k * 7 + 1) % n_pages);
        uint16_t *pool = malloc((size_t)(n_pages * H) * sizeof *pool);
        for (int64_t k = 0; k < n_pages * H; ++k) pool[k] = (uint16_t)(0x3000 + rnd() % 0x0c00);
        int32_t *ids = malloc((size_t)(T ? T : 1) * sizeof *ids);
        uint16_t *x = malloc((size_t)(T ? T * H : 1) * sizeof *x);
        float *yi = malloc((size_t)(T ? T * H : 1) * sizeof *yi);
        double *yo = malloc((size_t)(T ? T * H : 1) * sizeof *yo);
        for (int t = 0; t < T; ++t) ids[t] = (int32_t)(rnd() % (uint32_t)(n_ad + 1)) - 1;
        for (int k = 0; k < T * H; ++k) { x[k] = (uint16_t)(0x3800 + rnd() % 0x400); yi[k] = (float)(rnd() % 17) - 8.f; }
        int used = 0;
        REQUIRE(slo_lora_apply(pool, n_pages, H, dtype, rank, off, lists, n_ad, ids, T, x, yi, yo, 1 + (int)(rnd() % 3), &used) == 0);
        REQUIRE(used >= 1);
        for (int t = 0; t < T; ++t)
            if (ids[t] < 0 || rank[ids[t]] == 0)
                for (int d = 0; d < H; ++d) REQUIRE(yo[(size_t)t * H + d] == (double)yi[(size_t)t * H + d]);
        /* refused before anything is read: an adapter id and a page index out of range */
        if (T > 0) {
            const int32_t keep = ids[0];
            ids[0] = n_ad;
            REQUIRE(slo_lora_apply(pool, n_pages, H, dtype, rank, off, lists, n_ad, ids, T, x, yi, yo, 1, NULL) == -2);
            ids[0] = keep;
        }
        for (int t = 0; t < T; ++t)
            if (ids[t] >= 0 && rank[ids[t]] > 0) {
                const int32_t keep = lists[off[ids[t]]];
                lists[off[ids[t]]] = (int32_t)n_pages;
                REQUIRE(slo_lora_apply(pool, n_pages, H, dtype, rank, off, lists, n_ad, ids, T, x, yi, yo, 1, NULL) == -1);
                lists[off[ids[t]]] = keep;
                break;
            }
        /* gathers of one list, exact-size outputs */
        for (int a = 0; a < n_ad; ++a) {
            const int32_t r = rank[a];
            double *g = malloc((size_t)(r ? r * H : 1) * sizeof *g);
            uint16_t *gb = malloc((size_t)(r ? r * H : 1) * sizeof *gb);
            REQUIRE(slo_gather(pool, n_pages, H, dtype, lists + off[a], r, g) == 0);
            REQUIRE(slo_gather_bits(pool, n_pages, H, lists + off[a], r, gb) == 0);
            for (int32_t j = 0; j < r; ++j)
                REQUIRE(memcmp(gb + (size_t)j * H, pool + (size_t)lists[off[a] + j] * H, (size_t)H * 2) == 0);
            free(g); free(gb);
        }
        free(rank); free(off); free(lists); free(pool); free(ids); free(x); free(yi); free(yo);
    }
    printf("oracle_san OK\n");
    return 0;
}
