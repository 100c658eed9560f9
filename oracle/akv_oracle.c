/*
 * AlignedKV CPU oracle  --  TEST INFRASTRUCTURE, NOT A PRODUCT PATH.
 *
 * A plain, slow, step-by-step CPU writing of decode attention over a
 * precision-aligned KV cache (paper: sections "Precision Alignment Criterion",
 * "A Framework for Aligning Precision" (Rule 1, Rule 2), "Dynamic
 * Quantization", "Quantization of K-Cache", "Quantization of V-Cache", and the
 * three equations of "Runtime of AlignedKV": S = QK^T/sqrt(128), softmax, O = SV).
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may use this
 * file.  It shares no code, header, table or helper with the HIP library.
 *
 * Two kinds of arithmetic, on purpose:
 *   - the DECISION path (which bits are read) is integer arithmetic plus IEEE
 *     binary32 operations in one fixed order, so that every byte and every
 *     mask is reproducible on any IEEE machine;
 *   - the VALUE path (the attention numbers) is binary64 on the dequantised
 *     values.
 *
 * Parity pins (tests/test_oracle_*.py): pack/unpack exhaustive; truncation
 * error bound exhaustive; half->float conversion against numpy; K and V rules
 * against brute force over every level assignment and against the numerical
 * error bound they promise; top-k against an exact sort; force_level=2 against
 * textbook fp64 attention; out at mixed levels against a numpy fp64 attention
 * over operands rebuilt from the exported lvlK / appliedV masks.  The whole file
 * also runs under AddressSanitizer + UBSan (tests/test_oracle_sanitizers.py).
 * UNPINNED (the paper fixes no value): top-k size 32,
 * the score floor 2^-64, and the size of (out - fp16 attention) on synthetic data.
 *
 * Notation follows the paper: K, V, Q, S, O, K_colmax, O_est.  fp16 bit pattern
 * h = s|e4..e0|m9..m0 ("Precision Alignment in Floating-Point Addition": 1 sign,
 * 5 exponent, 10 mantissa bits).  "First 8 bits" = h>>8 (HI plane), "first 12"
 * adds (h>>4)&15 (MID plane), all 16 add h&15 (LO plane) ("Dynamic Quantization").
 * Level 0 / 1 / 2 = 8 / 12 / 16 bits read = 2 / 6 / 10 mantissa bits kept.
 *
 * Cache layout (the "data rearrangement" of the paper, one slice per precision
 * part, each contiguous):
 *   TB = 256 tokens per K block, NB = Ncap / TB.
 *   K_hi [b][h][blk][d][j]      u8, j = token % 256          (channel-major in a block)
 *   K_mid[b][h][blk][d][j/2]    u8, even token low nibble, odd token high nibble
 *   K_lo                        same shape and packing as K_mid
 *   V_hi [b][h][t][d]           u8                            (token-major)
 *   V_mid[b][h][t][d/2]         u8, even channel low nibble, odd channel high nibble
 *   V_lo                        same as V_mid
 *   colmax[b][h][d]             u16 = max over stored tokens of (h & 0x7fff)
 *   lens[b]                     i32 tokens stored for sequence b
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define AKVO_TB 256
#define AKVO_A_MIN (-64)
#define AKVO_NBUCKET 65

/* ---------- fp16 helpers -------------------------------------------------- */

/* exact value of a binary16 pattern as binary64 (finite patterns; Inf/NaN map
 * to +-Inf / NaN through the C library) */
static double half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 31;
    int m = h & 1023;
    double v;
    if (e == 0) v = ldexp((double)m, -24);
    else if (e == 31) v = m ? NAN : INFINITY;
    else v = ldexp((double)(1024 + m), e - 25);
    return sign ? -v : v;
}

static float half_to_float(uint16_t h) { return (float)half_to_double(h); } /* exact: 11-bit significand */

static uint32_t float_bits(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    return u;
}

static int float_exp_field(float f) { return (int)((float_bits(f) >> 23) & 0xFF); }

/* "Dynamic Quantization": read 16, the first 12, or the first 8 bits; the bits
 * not read are filled with 100... */
static uint16_t read_at_level(uint16_t h, int level)
{
    if (level >= 2) return h;
    if (level == 1) return (uint16_t)((h & 0xFFF0) | 0x0008);
    return (uint16_t)((h & 0xFF00) | 0x0080);
}

static uint16_t colmax_floor(uint16_t cm) { return cm < 0x0400 ? (uint16_t)0x0400 : cm; }

/* smallest level that keeps at least m mantissa bits (2 / 6 / 10 available) */
static int level_for_mantissa_bits(int m)
{
    if (m <= 2) return 0;
    if (m <= 6) return 1;
    return 2;
}

/* ---------- plane addressing --------------------------------------------- */

typedef struct {
    int B, Hkv, D, Ncap;
    uint8_t *k_hi, *k_mid, *k_lo, *v_hi, *v_mid, *v_lo;
} planes_t;

static size_t k_hi_index(const planes_t *p, int b, int h, int t, int d)
{
    int NB = p->Ncap / AKVO_TB;
    int blk = t / AKVO_TB, j = t % AKVO_TB;
    return ((((size_t)b * p->Hkv + h) * NB + blk) * p->D + d) * AKVO_TB + j;
}
static size_t k_nib_index(const planes_t *p, int b, int h, int t, int d)
{
    int NB = p->Ncap / AKVO_TB;
    int blk = t / AKVO_TB, j = t % AKVO_TB;
    return ((((size_t)b * p->Hkv + h) * NB + blk) * p->D + d) * (AKVO_TB / 2) + j / 2;
}
static size_t v_hi_index(const planes_t *p, int b, int h, int t, int d)
{
    return (((size_t)b * p->Hkv + h) * p->Ncap + t) * p->D + d;
}
static size_t v_nib_index(const planes_t *p, int b, int h, int t, int d)
{
    return (((size_t)b * p->Hkv + h) * p->Ncap + t) * (p->D / 2) + d / 2;
}

static void put_nibble(uint8_t *byte, int high, unsigned nib)
{
    if (high) *byte = (uint8_t)((*byte & 0x0F) | (nib << 4));
    else *byte = (uint8_t)((*byte & 0xF0) | nib);
}
static unsigned get_nibble(uint8_t byte, int high) { return high ? (byte >> 4) & 15u : byte & 15u; }

static void store_k(const planes_t *p, int b, int h, int t, int d, uint16_t x)
{
    p->k_hi[k_hi_index(p, b, h, t, d)] = (uint8_t)(x >> 8);
    put_nibble(&p->k_mid[k_nib_index(p, b, h, t, d)], t & 1, (x >> 4) & 15u);
    put_nibble(&p->k_lo[k_nib_index(p, b, h, t, d)], t & 1, x & 15u);
}
static uint16_t load_k(const planes_t *p, int b, int h, int t, int d)
{
    unsigned hi = p->k_hi[k_hi_index(p, b, h, t, d)];
    unsigned mid = get_nibble(p->k_mid[k_nib_index(p, b, h, t, d)], t & 1);
    unsigned lo = get_nibble(p->k_lo[k_nib_index(p, b, h, t, d)], t & 1);
    return (uint16_t)((hi << 8) | (mid << 4) | lo);
}
static void store_v(const planes_t *p, int b, int h, int t, int d, uint16_t x)
{
    p->v_hi[v_hi_index(p, b, h, t, d)] = (uint8_t)(x >> 8);
    put_nibble(&p->v_mid[v_nib_index(p, b, h, t, d)], d & 1, (x >> 4) & 15u);
    put_nibble(&p->v_lo[v_nib_index(p, b, h, t, d)], d & 1, x & 15u);
}
static uint16_t load_v(const planes_t *p, int b, int h, int t, int d)
{
    unsigned hi = p->v_hi[v_hi_index(p, b, h, t, d)];
    unsigned mid = get_nibble(p->v_mid[v_nib_index(p, b, h, t, d)], d & 1);
    unsigned lo = get_nibble(p->v_lo[v_nib_index(p, b, h, t, d)], d & 1);
    return (uint16_t)((hi << 8) | (mid << 4) | lo);
}

static int shape_ok(int B, int Hq, int Hkv, int D, int Ncap)
{
    return B > 0 && Hkv > 0 && Hq > 0 && Hq % Hkv == 0 && D > 0 && D % 2 == 0 && Ncap > 0 && Ncap % AKVO_TB == 0;
}

/* ---------- exported: scalar helpers (used by the pin tests) -------------- */

double akvo_half_to_double(uint16_t h) { return half_to_double(h); }
uint16_t akvo_read_at_level(uint16_t h, int level) { return read_at_level(h, level); }
int akvo_level_for_mantissa_bits(int m) { return level_for_mantissa_bits(m); }

/* ---------- exported: append ("Dynamic Quantization": the cache keeps every
 * fp16 bit; K_colmax is maintained while storing, "Quantization of K-Cache") -- */

/* k_new, v_new: [B][Hkv][n][D] fp16 bit patterns.  n_new: [B] tokens to take
 * from the front of each sequence's n rows, or NULL for all n.  A sequence whose
 * new length would exceed Ncap is left untouched.  Returns the number of such
 * sequences, or -1 on a bad shape. */
int akvo_append(int B, int Hkv, int D, int Ncap, uint8_t *k_hi, uint8_t *k_mid, uint8_t *k_lo, uint8_t *v_hi,
                uint8_t *v_mid, uint8_t *v_lo, uint16_t *colmax, int32_t *lens, const uint16_t *k_new,
                const uint16_t *v_new, const int32_t *n_new, int n)
{
    if (!shape_ok(B, Hkv, Hkv, D, Ncap) || n < 0) return -1;
    planes_t p = {B, Hkv, D, Ncap, k_hi, k_mid, k_lo, v_hi, v_mid, v_lo};
    int overflowed = 0;
    for (int b = 0; b < B; ++b) {
        int cnt = n_new ? n_new[b] : n;
        if (cnt < 0 || cnt > n) return -1;
        if (lens[b] + cnt > Ncap) {
            ++overflowed;
            continue;
        }
        for (int h = 0; h < Hkv; ++h)
            for (int i = 0; i < cnt; ++i) {
                int t = lens[b] + i;
                const uint16_t *krow = k_new + (((size_t)b * Hkv + h) * n + i) * D;
                const uint16_t *vrow = v_new + (((size_t)b * Hkv + h) * n + i) * D;
                for (int d = 0; d < D; ++d) {
                    store_k(&p, b, h, t, d, krow[d]);
                    store_v(&p, b, h, t, d, vrow[d]);
                    uint16_t mag = krow[d] & 0x7FFF; /* |k| as bits: integer order = magnitude order */
                    uint16_t *cm = &colmax[((size_t)b * Hkv + h) * D + d];
                    if (mag > *cm) *cm = mag;
                }
            }
        lens[b] += cnt;
    }
    return overflowed;
}

/* planes -> [B][Hkv][Ncap][D] fp16 bit patterns (all Ncap slots) */
int akvo_unpack(int B, int Hkv, int D, int Ncap, const uint8_t *k_hi, const uint8_t *k_mid, const uint8_t *k_lo,
                const uint8_t *v_hi, const uint8_t *v_mid, const uint8_t *v_lo, uint16_t *k_out, uint16_t *v_out)
{
    if (!shape_ok(B, Hkv, Hkv, D, Ncap)) return -1;
    planes_t p = {B,           Hkv, D, Ncap, (uint8_t *)k_hi, (uint8_t *)k_mid, (uint8_t *)k_lo, (uint8_t *)v_hi,
                  (uint8_t *)v_mid, (uint8_t *)v_lo};
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < Hkv; ++h)
            for (int t = 0; t < Ncap; ++t)
                for (int d = 0; d < D; ++d) {
                    size_t o = (((size_t)b * Hkv + h) * Ncap + t) * D + d;
                    k_out[o] = load_k(&p, b, h, t, d);
                    v_out[o] = load_v(&p, b, h, t, d);
                }
    return 0;
}

/* ---------- exported: decode attention ------------------------------------ */

typedef struct {
    /* every pointer may be NULL (not wanted) */
    uint8_t *lvlK;     /* [B][Hkv][D]        level each K column is read at           */
    float *logits;     /* [B][Hq][Ncap]      q . K~ accumulated in binary32, t < len  */
    int8_t *a;         /* [B][Hq][Ncap]      floor(log2 of the unnormalised weight)   */
    int32_t *sel;      /* [B][Hq][topk]      selected tokens ascending, -1 padded     */
    float *oest;       /* [B][Hq][D]         O_est (unnormalised)                     */
    int16_t *Ehat;     /* [B][Hkv][D]        result exponent bound used by Rule 2     */
    uint8_t *needV;    /* [B][Hkv][Ncap][D]  level each V element needs               */
    uint8_t *appliedV; /* [B][Hkv][Ncap]     level each V row is read at              */
    uint64_t *counts;  /* [9] elements: K read at L0,L1,L2; V rows*D read at L0,L1,L2; V need L0,L1,L2 */
} akvo_debug;

/* one (sequence, KV head) pair */
static void decode_one(const planes_t *p, int Hq, int b, int h, int len, const uint16_t *colmax,
                       const uint16_t *q /* [B][Hq][D] */, double scale, int topk, int guard_bits, int force_level,
                       double *out, const akvo_debug *dbg, uint64_t counts[9])
{
    const int D = p->D, Ncap = p->Ncap, Hkv = p->Hkv;
    const int G = Hq / Hkv;
    const size_t bh = (size_t)b * Hkv + h;

    uint8_t *lvlK = (uint8_t *)malloc((size_t)D);
    float *logit = (float *)malloc(sizeof(float) * (size_t)G * (len > 0 ? len : 1));
    int *a = (int *)malloc(sizeof(int) * (size_t)G * (len > 0 ? len : 1));
    float *phat = (float *)malloc(sizeof(float) * (size_t)G * (len > 0 ? len : 1));
    int *E = (int *)malloc(sizeof(int) * (size_t)G * D);
    int *Ehat = (int *)malloc(sizeof(int) * (size_t)D);
    int *Ahat = (int *)malloc(sizeof(int) * (size_t)(len > 0 ? len : 1));
    uint8_t *applied = (uint8_t *)malloc((size_t)(len > 0 ? len : 1));
    int *sel = (int *)malloc(sizeof(int) * (size_t)(topk > 0 ? topk : 1));
    double *s = (double *)malloc(sizeof(double) * (size_t)(len > 0 ? len : 1));

    /* --- K rule: Rule 1, addend alignment, from q and K_colmax --------------
     * The addend of column d is about q_d * K_colmax_d.  The coarsest addend
     * (largest exponent emax) has its last fp16 place at 2^(emax-10); an addend
     * with exponent e needs 10 - (emax - e) mantissa bits to reach that place
     * (+ guard_bits), and the K element inherits the addend's bit width.
     * K_colmax below the smallest normal fp16 (2^-14, also an all-zero column)
     * counts as 2^-14: the places of a subnormal are those of that exponent. */
    for (int d = 0; d < D; ++d) lvlK[d] = 0;
    for (int g = 0; g < G; ++g) {
        const uint16_t *qg = q + ((size_t)b * Hq + (size_t)h * G + g) * D;
        int emax = -1;
        for (int d = 0; d < D; ++d) {
            float P = half_to_float(qg[d]) * half_to_float(colmax_floor(colmax[bh * D + d]));
            if (P != 0.0f && float_exp_field(P) > emax) emax = float_exp_field(P);
        }
        for (int d = 0; d < D; ++d) {
            float P = half_to_float(qg[d]) * half_to_float(colmax_floor(colmax[bh * D + d]));
            int level = 0;
            if (P != 0.0f) level = level_for_mantissa_bits(10 + guard_bits - (emax - float_exp_field(P)));
            if (level > lvlK[d]) lvlK[d] = (uint8_t)level; /* query heads sharing the KV head: take the max */
        }
    }
    if (force_level >= 0)
        for (int d = 0; d < D; ++d) lvlK[d] = (uint8_t)force_level;
    if (dbg->lvlK) memcpy(dbg->lvlK + bh * D, lvlK, (size_t)D);
    for (int d = 0; d < D; ++d) counts[lvlK[d]] += (uint64_t)len;

    /* --- logits in binary32, channel order ascending (decision path) -------- */
    for (int g = 0; g < G; ++g) {
        const uint16_t *qg = q + ((size_t)b * Hq + (size_t)h * G + g) * D;
        for (int t = 0; t < len; ++t) {
            float acc = 0.0f;
            for (int d = 0; d < D; ++d) {
                float kq = half_to_float(read_at_level(load_k(p, b, h, t, d), lvlK[d]));
                acc = acc + half_to_float(qg[d]) * kq; /* product exact in binary32; one rounding per add */
            }
            logit[(size_t)g * len + t] = acc;
        }
    }

    /* --- score exponents: weight_t = 2^(x_t), x_t = (l_t - M) * scale*log2(e) */
    const float c = (float)(scale * 1.4426950408889634);
    for (int g = 0; g < G; ++g) {
        if (len == 0) break;
        float M = logit[(size_t)g * len];
        for (int t = 1; t < len; ++t)
            if (logit[(size_t)g * len + t] > M) M = logit[(size_t)g * len + t];
        for (int t = 0; t < len; ++t) {
            float diff = logit[(size_t)g * len + t] - M;
            float x = diff * c;
            float fl = floorf(x);
            int at = (fl < (float)AKVO_A_MIN) ? AKVO_A_MIN : (int)fl;
            float f = x - fl;
            a[(size_t)g * len + t] = at;
            phat[(size_t)g * len + t] = ldexpf(1.0f + f, at); /* piecewise-linear 2^x, floor at 2^-64 */
        }
    }

    /* --- approximate top-k by exponent bucket, O_est, result exponents ------ */
    for (int d = 0; d < D; ++d) Ehat[d] = 32767;
    for (int g = 0; g < G; ++g) {
        const size_t hq = (size_t)b * Hq + (size_t)h * G + g;
        int kk = topk < len ? topk : len;
        int cnt[AKVO_NBUCKET];
        for (int j = 0; j < AKVO_NBUCKET; ++j) cnt[j] = 0;
        for (int t = 0; t < len; ++t) cnt[-a[(size_t)g * len + t]]++;
        int J = 0, below = 0; /* below = tokens in buckets < J */
        while (kk > 0 && below + cnt[J] < kk) below += cnt[J++];
        int nsel = 0, from_cut = kk - below;
        for (int t = 0; t < len && nsel < kk; ++t) {
            int j = -a[(size_t)g * len + t];
            if (j < J) sel[nsel++] = t;
            else if (j == J && from_cut > 0) {
                sel[nsel++] = t;
                --from_cut;
            }
        }
        for (int d = 0; d < D; ++d) {
            float acc = 0.0f;
            for (int i = 0; i < nsel; ++i)
                acc = fmaf(phat[(size_t)g * len + sel[i]], half_to_float(load_v(p, b, h, sel[i], d)), acc);
            E[(size_t)g * D + d] = float_exp_field(acc) - 127;
            if (dbg->oest) dbg->oest[hq * D + d] = acc;
            if (E[(size_t)g * D + d] < Ehat[d]) Ehat[d] = E[(size_t)g * D + d];
        }
        if (dbg->sel)
            for (int i = 0; i < topk; ++i) dbg->sel[hq * topk + i] = i < nsel ? sel[i] : -1;
        if (dbg->logits)
            for (int t = 0; t < len; ++t) dbg->logits[hq * Ncap + t] = logit[(size_t)g * len + t];
        if (dbg->a)
            for (int t = 0; t < len; ++t) dbg->a[hq * Ncap + t] = (int8_t)a[(size_t)g * len + t];
    }
    if (dbg->Ehat)
        for (int d = 0; d < D; ++d) dbg->Ehat[bh * D + d] = (int16_t)Ehat[d];

    /* --- V rule: Rule 2, result alignment, against O_est --------------------
     * The result of channel d has its last fp16 place at 2^(Ehat_d - 10).  The
     * addend weight_t * v has exponent about tau = Ahat_t + (ev' - 15); it needs
     * 10 - (Ehat_d - tau) mantissa bits (+ guard_bits).  ev' = max(ev, 1): a
     * subnormal's places are those of the smallest normal exponent. */
    for (int t = 0; t < len; ++t) {
        int am = a[t];
        for (int g = 1; g < G; ++g)
            if (a[(size_t)g * len + t] > am) am = a[(size_t)g * len + t];
        Ahat[t] = am;
        int row = 0;
        for (int d = 0; d < D; ++d) {
            int ev = (p->v_hi[v_hi_index(p, b, h, t, d)] >> 2) & 31;
            if (ev < 1) ev = 1;
            int tau = Ahat[t] + ev - 15;
            int need = level_for_mantissa_bits(10 + guard_bits - (Ehat[d] - tau));
            if (force_level >= 0) need = force_level;
            if (dbg->needV) dbg->needV[(bh * Ncap + t) * D + d] = (uint8_t)need;
            counts[6 + need]++;
            if (need > row) row = need;
        }
        applied[t] = (uint8_t)row; /* the fetch granule is one token row */
        counts[3 + row] += (uint64_t)D;
        if (dbg->appliedV) dbg->appliedV[bh * Ncap + t] = (uint8_t)row;
    }

    /* --- value path in binary64: S = QK~^T * scale, softmax, O = S V~ ------- */
    for (int g = 0; g < G; ++g) {
        const size_t hq = (size_t)b * Hq + (size_t)h * G + g;
        const uint16_t *qg = q + hq * D;
        for (int d = 0; d < D; ++d) out[hq * D + d] = 0.0;
        if (len == 0) continue;
        double mx = -INFINITY;
        for (int t = 0; t < len; ++t) {
            double acc = 0.0;
            for (int d = 0; d < D; ++d)
                acc += half_to_double(qg[d]) * half_to_double(read_at_level(load_k(p, b, h, t, d), lvlK[d]));
            s[t] = acc * scale;
            if (s[t] > mx) mx = s[t];
        }
        double Z = 0.0;
        for (int t = 0; t < len; ++t) {
            s[t] = exp(s[t] - mx);
            Z += s[t];
        }
        for (int d = 0; d < D; ++d) {
            double acc = 0.0;
            for (int t = 0; t < len; ++t)
                acc += s[t] * half_to_double(read_at_level(load_v(p, b, h, t, d), applied[t]));
            out[hq * D + d] = acc / Z;
        }
    }

    free(lvlK);
    free(logit);
    free(a);
    free(phat);
    free(E);
    free(Ehat);
    free(Ahat);
    free(applied);
    free(sel);
    free(s);
}

/* q: [B][Hq][D] fp16 bits.  out: [B][Hq][D] binary64.  scale <= 0 means
 * 1/sqrt(D).  force_level: -1 adaptive; 0/1/2 every element read at that level
 * (2 = the paper's control group, always 16 bits).  Returns 0, or -1 on bad
 * arguments. */
int akvo_decode_attention(int B, int Hq, int Hkv, int D, int Ncap, const uint8_t *k_hi, const uint8_t *k_mid,
                          const uint8_t *k_lo, const uint8_t *v_hi, const uint8_t *v_mid, const uint8_t *v_lo,
                          const uint16_t *colmax, const int32_t *lens, const uint16_t *q, float scale, int topk,
                          int guard_bits, int force_level, double *out, const akvo_debug *dbg_in)
{
    if (!shape_ok(B, Hq, Hkv, D, Ncap) || topk < 1 || force_level < -1 || force_level > 2) return -1;
    for (int b = 0; b < B; ++b)
        if (lens[b] < 0 || lens[b] > Ncap) return -1;
    akvo_debug none;
    memset(&none, 0, sizeof none);
    const akvo_debug *dbg = dbg_in ? dbg_in : &none;
    const double scale_d = scale > 0.0f ? (double)scale : 1.0 / sqrt((double)D);
    planes_t p = {B,           Hkv, D, Ncap, (uint8_t *)k_hi, (uint8_t *)k_mid, (uint8_t *)k_lo, (uint8_t *)v_hi,
                  (uint8_t *)v_mid, (uint8_t *)v_lo};
    uint64_t total[9] = {0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma omp parallel for schedule(dynamic, 1)
    for (int bh = 0; bh < B * Hkv; ++bh) {
        uint64_t counts[9] = {0, 0, 0, 0, 0, 0, 0, 0, 0};
        decode_one(&p, Hq, bh / Hkv, bh % Hkv, lens[bh / Hkv], colmax, q, scale_d, topk, guard_bits, force_level, out,
                   dbg, counts);
#pragma omp critical
        for (int i = 0; i < 9; ++i) total[i] += counts[i];
    }
    if (dbg->counts)
        for (int i = 0; i < 9; ++i) dbg->counts[i] = total[i];
    return 0;
}

/* Textbook attention in binary64 on plain fp16 tensors k, v: [B][Hkv][Ncap][D]
 * ("Runtime of AlignedKV": S = QK^T/sqrt(128); softmax; O = SV). */
int akvo_fp16_attention(int B, int Hq, int Hkv, int D, int Ncap, const uint16_t *k, const uint16_t *v,
                        const int32_t *lens, const uint16_t *q, float scale, double *out)
{
    if (!shape_ok(B, Hq, Hkv, D, Ncap)) return -1;
    const double scale_d = scale > 0.0f ? (double)scale : 1.0 / sqrt((double)D);
    const int G = Hq / Hkv;
#pragma omp parallel for schedule(dynamic, 1)
    for (int bq = 0; bq < B * Hq; ++bq) {
        int b = bq / Hq, hq = bq % Hq, h = hq / G, len = lens[b];
        const uint16_t *qg = q + (size_t)bq * D;
        const uint16_t *kk = k + ((size_t)b * Hkv + h) * Ncap * D;
        const uint16_t *vv = v + ((size_t)b * Hkv + h) * Ncap * D;
        for (int d = 0; d < D; ++d) out[(size_t)bq * D + d] = 0.0;
        if (len <= 0) continue;
        double *s = (double *)malloc(sizeof(double) * (size_t)len);
        double mx = -INFINITY, Z = 0.0;
        for (int t = 0; t < len; ++t) {
            double acc = 0.0;
            for (int d = 0; d < D; ++d) acc += half_to_double(qg[d]) * half_to_double(kk[(size_t)t * D + d]);
            s[t] = acc * scale_d;
            if (s[t] > mx) mx = s[t];
        }
        for (int t = 0; t < len; ++t) {
            s[t] = exp(s[t] - mx);
            Z += s[t];
        }
        for (int d = 0; d < D; ++d) {
            double acc = 0.0;
            for (int t = 0; t < len; ++t) acc += s[t] * half_to_double(vv[(size_t)t * D + d]);
            out[(size_t)bq * D + d] = acc / Z;
        }
        free(s);
    }
    return 0;
}

/* ---------- exported: what other fetch granules would read (studies, no kernel reads the cache that way) -------
 * "Dynamic Quantization" (data re-arrangement): the hardware reads in units of several bytes, so the level that is
 * applied is the maximum of the per-element needs over a fetch unit.  The cache's unit for V is one token row
 * (1 token x D channels).  This function answers what a unit of tt tokens x cc channels would read instead.
 * needV: [B][Hkv][Ncap][D] per-element levels as akvo_decode_attention exports them; tt divides 256, cc divides D.
 * counts[l] = V elements (of tokens t < lens[b]) that would be read at level l.  Returns 0, or -1 on bad arguments. */
int akvo_v_granule_counts(int B, int Hkv, int D, int Ncap, const uint8_t *needV, const int32_t *lens, int tt, int cc,
                          uint64_t counts[3])
{
    if (!shape_ok(B, Hkv, Hkv, D, Ncap) || tt < 1 || cc < 1 || AKVO_TB % tt != 0 || D % cc != 0) return -1;
    counts[0] = counts[1] = counts[2] = 0;
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < Hkv; ++h)
            for (int t0 = 0; t0 < lens[b]; t0 += tt)
                for (int d0 = 0; d0 < D; d0 += cc) {
                    int lvl = 0, ntok = 0;
                    for (int t = t0; t < t0 + tt && t < lens[b]; ++t) {
                        ++ntok;
                        for (int d = d0; d < d0 + cc; ++d) {
                            int need = needV[((((size_t)b * Hkv + h) * Ncap) + t) * D + d];
                            if (need > lvl) lvl = need;
                        }
                    }
                    counts[lvl] += (uint64_t)ntok * (uint64_t)cc;
                }
    return 0;
}

/* Rule 1 with one column maximum per `block` tokens instead of one per sequence ("Quantization of K-Cache": the
 * data within a column are only relatively similar).  For every block of `block` tokens (block a multiple of 1,
 * blocks start at token 0) the column maxima are taken over the tokens of that block only, and the K rule of
 * akvo_decode_attention is applied with them: coarsest addend and every addend bounded inside the block.
 * lvl_out: [B][Hkv][ceil(Ncap / block)][D] levels per (block, column), or NULL; counts[l] = K elements (tokens
 * t < lens[b]) read at level l.  A block >= the sequence reproduces lvlK of akvo_decode_attention. */
int akvo_k_levels_per_block(int B, int Hq, int Hkv, int D, int Ncap, const uint8_t *k_hi, const uint8_t *k_mid,
                            const uint8_t *k_lo, const int32_t *lens, const uint16_t *q, int guard_bits, int block,
                            uint8_t *lvl_out, uint64_t counts[3])
{
    if (!shape_ok(B, Hq, Hkv, D, Ncap) || block < 1) return -1;
    planes_t p = {B, Hkv, D, Ncap, (uint8_t *)k_hi, (uint8_t *)k_mid, (uint8_t *)k_lo, NULL, NULL, NULL};
    const int G = Hq / Hkv;
    const int nblk_cap = (Ncap + block - 1) / block;
    counts[0] = counts[1] = counts[2] = 0;
    uint16_t *cm = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)D);
    uint8_t *lvl = (uint8_t *)malloc((size_t)D);
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < Hkv; ++h)
            for (int t0 = 0, bi = 0; t0 < lens[b]; t0 += block, ++bi) {
                int t1 = t0 + block < lens[b] ? t0 + block : lens[b];
                for (int d = 0; d < D; ++d) {
                    cm[d] = 0;
                    for (int t = t0; t < t1; ++t) {
                        uint16_t mag = load_k(&p, b, h, t, d) & 0x7FFF;
                        if (mag > cm[d]) cm[d] = mag;
                    }
                    lvl[d] = 0;
                }
                for (int g = 0; g < G; ++g) {
                    const uint16_t *qg = q + ((size_t)b * Hq + (size_t)h * G + g) * D;
                    int emax = -1;
                    for (int d = 0; d < D; ++d) {
                        float P = half_to_float(qg[d]) * half_to_float(colmax_floor(cm[d]));
                        if (P != 0.0f && float_exp_field(P) > emax) emax = float_exp_field(P);
                    }
                    for (int d = 0; d < D; ++d) {
                        float P = half_to_float(qg[d]) * half_to_float(colmax_floor(cm[d]));
                        int level = 0;
                        if (P != 0.0f) level = level_for_mantissa_bits(10 + guard_bits - (emax - float_exp_field(P)));
                        if (level > lvl[d]) lvl[d] = (uint8_t)level;
                    }
                }
                for (int d = 0; d < D; ++d) {
                    counts[lvl[d]] += (uint64_t)(t1 - t0);
                    if (lvl_out) lvl_out[((((size_t)b * Hkv + h) * nblk_cap) + bi) * D + d] = lvl[d];
                }
            }
    free(cm);
    free(lvl);
    return 0;
}

int akvo_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* number of threads the parallel loops over (sequence, head) use from now on (timing at one thread and at all) */
void akvo_set_threads(int n)
{
#ifdef _OPENMP
    if (n >= 1) omp_set_num_threads(n);
#else
    (void)n;
#endif
}
