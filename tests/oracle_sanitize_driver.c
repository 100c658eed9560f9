/*
 * Drives every exported function of the two CPU oracles (oracle/akv_oracle.c, oracle/akw_oracle.c) on buffers of
 * exactly the documented sizes, so that a build with -fsanitize=address,undefined reports any access outside them and
 * any undefined operation (shift, signed overflow, misaligned access).  Built and run by tests/test_oracle_sanitizers.py;
 * test infrastructure only.  Exit status 0 = ran clean.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    uint8_t *lvlK;
    float *logits;
    int8_t *a;
    int32_t *sel;
    float *oest;
    int16_t *Ehat;
    uint8_t *needV;
    uint8_t *appliedV;
    uint64_t *counts;
} akvo_debug;

int akvo_append(int B, int Hkv, int D, int Ncap, uint8_t *k_hi, uint8_t *k_mid, uint8_t *k_lo, uint8_t *v_hi,
                uint8_t *v_mid, uint8_t *v_lo, uint16_t *colmax, int32_t *lens, const uint16_t *k_new,
                const uint16_t *v_new, const int32_t *n_new, int n);
int akvo_unpack(int B, int Hkv, int D, int Ncap, const uint8_t *k_hi, const uint8_t *k_mid, const uint8_t *k_lo,
                const uint8_t *v_hi, const uint8_t *v_mid, const uint8_t *v_lo, uint16_t *k_out, uint16_t *v_out);
int akvo_decode_attention(int B, int Hq, int Hkv, int D, int Ncap, const uint8_t *k_hi, const uint8_t *k_mid,
                          const uint8_t *k_lo, const uint8_t *v_hi, const uint8_t *v_mid, const uint8_t *v_lo,
                          const uint16_t *colmax, const int32_t *lens, const uint16_t *q, float scale, int topk,
                          int guard_bits, int force_level, double *out, const akvo_debug *dbg_in);
int akvo_fp16_attention(int B, int Hq, int Hkv, int D, int Ncap, const uint16_t *k, const uint16_t *v,
                        const int32_t *lens, const uint16_t *q, float scale, double *out);
int akvo_v_granule_counts(int B, int Hkv, int D, int Ncap, const uint8_t *needV, const int32_t *lens, int tt, int cc,
                          uint64_t counts[3]);
int akvo_k_levels_per_block(int B, int Hq, int Hkv, int D, int Ncap, const uint8_t *k_hi, const uint8_t *k_mid,
                            const uint8_t *k_lo, const int32_t *lens, const uint16_t *q, int guard_bits, int block,
                            uint8_t *lvl_out, uint64_t counts[3]);
double akvo_half_to_double(uint16_t h);
uint16_t akvo_read_at_level(uint16_t h, int level);
int akvo_level_for_mantissa_bits(int m);

int akwo_pack(int K, int N, const uint16_t *W, uint8_t *hi, uint8_t *mid, uint8_t *lo, uint16_t *rowmax);
int akwo_unpack(int K, int N, const uint8_t *hi, const uint8_t *mid, const uint8_t *lo, uint16_t *W_out);
int akwo_levels(int B, int K, const uint16_t *x, const uint16_t *rowmax, int guard_bits, int force_level, uint8_t *lvl);
int akwo_gemv(int B, int K, int N, const uint8_t *hi, const uint8_t *mid, const uint8_t *lo, const uint16_t *rowmax,
              const uint16_t *x, int guard_bits, int force_level, double *y, uint8_t *lvl_out, double *abs_sum);
double akwo_half_to_double(uint16_t h);
uint16_t akwo_read_at_level(uint16_t h, int level);

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd(void)
{
    rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull;
    return (uint32_t)(rng_state >> 33);
}
/* a finite fp16 pattern: any sign and mantissa, exponent field 0..30 (subnormals and zeros included) */
static uint16_t finite_half(int emin, int emax)
{
    uint32_t r = rnd();
    uint32_t e = (uint32_t)emin + (rnd() % (uint32_t)(emax - emin + 1));
    return (uint16_t)(((r & 1u) << 15) | (e << 10) | ((r >> 1) & 1023u));
}
static void *exact(size_t bytes) /* an allocation of exactly this size, zeroed */
{
    void *p = calloc(bytes ? bytes : 1, 1);
    if (!p) exit(3);
    return p;
}
#define CHECK(c)                                                          \
    do {                                                                  \
        if (!(c)) {                                                       \
            fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #c); \
            exit(2);                                                      \
        }                                                                 \
    } while (0)

static void kv_case(int B, int Hq, int Hkv, int Ncap, const int *len_list, int topk, int guard, int force)
{
    const int D = 128, NB = Ncap / 256;
    size_t bh = (size_t)B * Hkv;
    uint8_t *k_hi = exact(bh * NB * D * 256), *k_mid = exact(bh * NB * D * 128), *k_lo = exact(bh * NB * D * 128);
    uint8_t *v_hi = exact(bh * Ncap * D), *v_mid = exact(bh * Ncap * D / 2), *v_lo = exact(bh * Ncap * D / 2);
    uint16_t *colmax = exact(bh * D * 2);
    int32_t *lens = exact((size_t)B * 4), *n_new = exact((size_t)B * 4);
    int n = 0;
    for (int b = 0; b < B; ++b) {
        n_new[b] = len_list[b];
        if (len_list[b] > n) n = len_list[b];
    }
    uint16_t *k_new = exact(bh * (size_t)n * D * 2), *v_new = exact(bh * (size_t)n * D * 2);
    for (size_t i = 0; i < bh * (size_t)n * D; ++i) {
        k_new[i] = finite_half(0, 24);
        v_new[i] = finite_half(0, 24);
    }
    /* in two calls, the second ragged; then one call that must be refused for capacity */
    int32_t *first = exact((size_t)B * 4), *second = exact((size_t)B * 4);
    for (int b = 0; b < B; ++b) {
        first[b] = n_new[b] / 2;
        second[b] = n_new[b] - first[b];
    }
    CHECK(akvo_append(B, Hkv, D, Ncap, k_hi, k_mid, k_lo, v_hi, v_mid, v_lo, colmax, lens, k_new, v_new, first, n) == 0);
    {   /* the second call takes its rows from the front of a fresh array */
        uint16_t *k2 = exact(bh * (size_t)n * D * 2), *v2 = exact(bh * (size_t)n * D * 2);
        for (size_t i = 0; i < bh * (size_t)n * D; ++i) {
            k2[i] = finite_half(0, 24);
            v2[i] = finite_half(0, 24);
        }
        CHECK(akvo_append(B, Hkv, D, Ncap, k_hi, k_mid, k_lo, v_hi, v_mid, v_lo, colmax, lens, k2, v2, second, n) == 0);
        free(k2);
        free(v2);
    }
    for (int b = 0; b < B; ++b) CHECK(lens[b] == len_list[b]);
    {
        int32_t *too_many = exact((size_t)B * 4);
        int expect = 0;
        for (int b = 0; b < B; ++b) {
            too_many[b] = n;
            if (lens[b] + n > Ncap) ++expect;
        }
        int32_t *saved = exact((size_t)B * 4);
        memcpy(saved, lens, (size_t)B * 4);
        int refused = akvo_append(B, Hkv, D, Ncap, k_hi, k_mid, k_lo, v_hi, v_mid, v_lo, colmax, lens, k_new, v_new,
                                  too_many, n);
        CHECK(refused == expect);
        /* back to the lengths of len_list: rows beyond lens are ignored by every reader (K_colmax keeps the extra
         * rows' maxima, which is harmless here: nothing below compares values) */
        memcpy(lens, saved, (size_t)B * 4);
        free(too_many);
        free(saved);
    }
    uint16_t *q = exact((size_t)B * Hq * D * 2);
    for (size_t i = 0; i < (size_t)B * Hq * D; ++i) q[i] = finite_half(8, 18);
    double *out = exact((size_t)B * Hq * D * 8);
    uint64_t counts[9];
    akvo_debug dbg = {exact(bh * D),
                      exact((size_t)B * Hq * Ncap * 4),
                      exact((size_t)B * Hq * Ncap),
                      exact((size_t)B * Hq * topk * 4),
                      exact((size_t)B * Hq * D * 4),
                      exact(bh * D * 2),
                      exact(bh * (size_t)Ncap * D),
                      exact(bh * Ncap),
                      counts};
    CHECK(akvo_decode_attention(B, Hq, Hkv, D, Ncap, k_hi, k_mid, k_lo, v_hi, v_mid, v_lo, colmax, lens, q, 0.0f, topk,
                                guard, force, out, &dbg) == 0);
    CHECK(akvo_decode_attention(B, Hq, Hkv, D, Ncap, k_hi, k_mid, k_lo, v_hi, v_mid, v_lo, colmax, lens, q, 0.25f, topk,
                                guard, force, out, NULL) == 0);
    {   /* the granule studies on the exported needs and on the K planes */
        uint64_t gc[3];
        CHECK(akvo_v_granule_counts(B, Hkv, D, Ncap, dbg.needV, lens, 1, D, gc) == 0);
        CHECK(akvo_v_granule_counts(B, Hkv, D, Ncap, dbg.needV, lens, 4, 32, gc) == 0);
        CHECK(akvo_v_granule_counts(B, Hkv, D, Ncap, dbg.needV, lens, 256, 1, gc) == 0);
        CHECK(akvo_v_granule_counts(B, Hkv, D, Ncap, dbg.needV, lens, 3, 32, gc) == -1);
        const int block = 64, nb = (Ncap + block - 1) / block;
        uint8_t *lv = exact(bh * (size_t)nb * D);
        CHECK(akvo_k_levels_per_block(B, Hq, Hkv, D, Ncap, k_hi, k_mid, k_lo, lens, q, guard, block, lv, gc) == 0);
        CHECK(akvo_k_levels_per_block(B, Hq, Hkv, D, Ncap, k_hi, k_mid, k_lo, lens, q, guard, Ncap, NULL, gc) == 0);
        free(lv);
    }
    uint16_t *k_out = exact(bh * (size_t)Ncap * D * 2), *v_out = exact(bh * (size_t)Ncap * D * 2);
    CHECK(akvo_unpack(B, Hkv, D, Ncap, k_hi, k_mid, k_lo, v_hi, v_mid, v_lo, k_out, v_out) == 0);
    CHECK(akvo_fp16_attention(B, Hq, Hkv, D, Ncap, k_out, v_out, lens, q, 0.0f, out) == 0);
    /* refused arguments return an error and touch nothing */
    CHECK(akvo_decode_attention(B, Hq, Hkv, D, Ncap + 1, k_hi, k_mid, k_lo, v_hi, v_mid, v_lo, colmax, lens, q, 0.0f,
                                topk, guard, force, out, NULL) == -1);
    CHECK(akvo_decode_attention(B, Hq, Hkv, D, Ncap, k_hi, k_mid, k_lo, v_hi, v_mid, v_lo, colmax, lens, q, 0.0f, 0,
                                guard, force, out, NULL) == -1);
    free(k_hi); free(k_mid); free(k_lo); free(v_hi); free(v_mid); free(v_lo); free(colmax); free(lens); free(n_new);
    free(k_new); free(v_new); free(first); free(second); free(q); free(out); free(k_out); free(v_out);
    free(dbg.lvlK); free(dbg.logits); free(dbg.a); free(dbg.sel); free(dbg.oest); free(dbg.Ehat); free(dbg.needV);
    free(dbg.appliedV);
}

static void weight_case(int B, int K, int N, int guard, int force)
{
    uint16_t *W = exact((size_t)K * N * 2), *W2 = exact((size_t)K * N * 2), *x = exact((size_t)B * K * 2);
    for (size_t i = 0; i < (size_t)K * N; ++i) W[i] = finite_half(0, 20);
    for (size_t i = 0; i < (size_t)B * K; ++i) x[i] = finite_half(0, 22);
    uint8_t *hi = exact((size_t)K * N), *mid = exact((size_t)K * N / 2), *lo = exact((size_t)K * N / 2);
    uint16_t *rowmax = exact((size_t)K * 2);
    uint8_t *lvl = exact((size_t)K);
    double *y = exact((size_t)B * N * 8), *sa = exact((size_t)B * N * 8);
    CHECK(akwo_pack(K, N, W, hi, mid, lo, rowmax) == 0);
    CHECK(akwo_unpack(K, N, hi, mid, lo, W2) == 0);
    CHECK(memcmp(W, W2, (size_t)K * N * 2) == 0);
    CHECK(akwo_levels(B, K, x, rowmax, guard, force, lvl) == 0);
    CHECK(akwo_gemv(B, K, N, hi, mid, lo, rowmax, x, guard, force, y, lvl, sa) == 0);
    CHECK(akwo_gemv(B, K, N, hi, mid, lo, rowmax, x, guard, force, y, NULL, NULL) == 0);
    free(W); free(W2); free(x); free(hi); free(mid); free(lo); free(rowmax); free(lvl); free(y); free(sa);
}

int main(void)
{
    for (uint32_t h = 0; h < 65536; ++h) {
        (void)akvo_half_to_double((uint16_t)h);
        (void)akwo_half_to_double((uint16_t)h);
        for (int l = 0; l < 3; ++l) CHECK(akvo_read_at_level((uint16_t)h, l) == akwo_read_at_level((uint16_t)h, l));
    }
    for (int m = -40; m <= 40; ++m) (void)akvo_level_for_mantissa_bits(m);
    {   /* MHA: a full sequence, a ragged one, an empty one, a single token */
        int lens[4] = {512, 301, 0, 1};
        kv_case(4, 2, 2, 512, lens, 32, 0, -1);
        kv_case(4, 2, 2, 512, lens, 64, 2, -1);
        for (int f = 0; f < 3; ++f) kv_case(4, 2, 2, 512, lens, 1, 0, f);
    }
    {   /* groups of 4 query heads; fewer tokens than the top-k */
        int lens[2] = {257, 7};
        kv_case(2, 8, 2, 512, lens, 32, 1, -1);
    }
    weight_case(1, 130, 64, 0, -1);
    weight_case(3, 64, 130, 2, -1);
    for (int f = 0; f < 3; ++f) weight_case(2, 33, 32, 0, f);
    printf("oracle sanitizer drive: clean\n");
    return 0;
}
