/*
 * Precision-aligned weight GEMV, CPU oracle  --  TEST INFRASTRUCTURE, NOT A PRODUCT PATH.
 *
 * The second workload of the precision-alignment framework: y = x W with the
 * weights W as the quantised operand ("Precision Alignment in Uncertainty
 * Calculation": A W = A (W_quant +- dW); "A Framework for Aligning Precision":
 * the framework proposes a precision for every parameter of the weights as well
 * as of the KV cache, and the bit width of an addend is the bit width of the
 * weight it comes from).  The result y is not known before the product, and no
 * cheap estimate of it exists, so the addends are aligned with each other:
 * Rule 1, exactly as for the K cache, with the roles
 *     channel d of K   <->  input feature k (row k of W),
 *     token t          <->  output feature n (column n of W),
 *     q                <->  the activation row x,
 *     K_colmax[d]      <->  rowmax[k] = max_n |W[k][n]|.
 * Storage and read-out follow "Dynamic Quantization": all 16 bits are kept in
 * three planes (first 8 / next 4 / last 4 bits), a row is read at 8, 12 or 16
 * bits, the bits not read count as 100...
 *
 * Only tests, the smoke check and a benchmark's CPU leg may use this file.  It
 * shares no code, header, table or helper with the HIP library.
 *
 * Decision path (levels): integer arithmetic plus IEEE binary32 products (exact:
 * two 11-bit significands).  Value path (y): binary64 on the dequantised values,
 * summed in ascending k.
 *
 * Parity pins (tests/test_oracle_weights.py): pack/unpack exhaustive over all
 * fp16 patterns; the three read-outs against values written out by hand; the
 * level rule against brute force over every level assignment and against the
 * error bound it promises; force_level = 2 against numpy's fp64 product;
 * invariance under power-of-two rescaling; monotone in guard_bits; several
 * activation rows take the maximum.  UNPINNED: nothing the paper prints -- the
 * paper names this use and gives no numbers for it.
 *
 * Layout (row-major in k, so that everything a row needs at its level is
 * contiguous):
 *   W_hi [k][n]     u8   h >> 8
 *   W_mid[k][n/2]   u8   (h >> 4) & 15, even column low nibble, odd column high nibble
 *   W_lo [k][n/2]   u8   h & 15, same packing
 *   rowmax[k]       u16  max over n of (h & 0x7fff)
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

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

static float half_to_float(uint16_t h) { return (float)half_to_double(h); } /* exact */

static int float_exp_field(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    return (int)((u >> 23) & 0xFF);
}

/* "Dynamic Quantization": 16, the first 12 or the first 8 bits; the rest reads as 100... */
static uint16_t read_at_level(uint16_t h, int level)
{
    if (level >= 2) return h;
    if (level == 1) return (uint16_t)((h & 0xFFF0) | 0x0008);
    return (uint16_t)((h & 0xFF00) | 0x0080);
}

/* smallest level that keeps at least m mantissa bits (2 / 6 / 10 available) */
static int level_for_mantissa_bits(int m)
{
    if (m <= 2) return 0;
    if (m <= 6) return 1;
    return 2;
}

static int shape_ok(int K, int N) { return K >= 1 && N >= 2 && N % 2 == 0; }

static uint16_t load_w(int N, const uint8_t *hi, const uint8_t *mid, const uint8_t *lo, int k, int n)
{
    size_t i = (size_t)k * N + n, j = (size_t)k * (N / 2) + n / 2;
    unsigned m = (n & 1) ? (mid[j] >> 4) & 15u : mid[j] & 15u;
    unsigned l = (n & 1) ? (lo[j] >> 4) & 15u : lo[j] & 15u;
    return (uint16_t)(((unsigned)hi[i] << 8) | (m << 4) | l);
}

/* W: [K][N] fp16 bit patterns -> planes and rowmax */
int akwo_pack(int K, int N, const uint16_t *W, uint8_t *hi, uint8_t *mid, uint8_t *lo, uint16_t *rowmax)
{
    if (!shape_ok(K, N)) return -1;
    for (int k = 0; k < K; ++k) {
        uint16_t mx = 0;
        for (int n = 0; n < N; n += 2) {
            uint16_t a = W[(size_t)k * N + n], b = W[(size_t)k * N + n + 1];
            hi[(size_t)k * N + n] = (uint8_t)(a >> 8);
            hi[(size_t)k * N + n + 1] = (uint8_t)(b >> 8);
            mid[(size_t)k * (N / 2) + n / 2] = (uint8_t)(((a >> 4) & 15u) | (((b >> 4) & 15u) << 4));
            lo[(size_t)k * (N / 2) + n / 2] = (uint8_t)((a & 15u) | ((b & 15u) << 4));
            if ((a & 0x7FFF) > mx) mx = a & 0x7FFF; /* integer order of the magnitude bits is magnitude order */
            if ((b & 0x7FFF) > mx) mx = b & 0x7FFF;
        }
        rowmax[k] = mx;
    }
    return 0;
}

int akwo_unpack(int K, int N, const uint8_t *hi, const uint8_t *mid, const uint8_t *lo, uint16_t *W_out)
{
    if (!shape_ok(K, N)) return -1;
    for (int k = 0; k < K; ++k)
        for (int n = 0; n < N; ++n) W_out[(size_t)k * N + n] = load_w(N, hi, mid, lo, k, n);
    return 0;
}

/* Rule 1 for the rows of W.  For the activation row b the addend of input feature k is about
 * x[b][k] * rowmax[k]; the coarsest addend (largest exponent emax_b) has its last fp16 place at
 * 2^(emax_b - 10); an addend with exponent e needs 10 - (emax_b - e) mantissa bits to reach that
 * place (+ guard_bits), and the weight inherits the addend's bit width.  A rowmax below the
 * smallest normal fp16 counts as 2^-14.  A row of W is read once for all activation rows: the
 * maximum over b.  lvl: [K]. */
int akwo_levels(int B, int K, const uint16_t *x, const uint16_t *rowmax, int guard_bits, int force_level, uint8_t *lvl)
{
    if (B < 1 || K < 1) return -1;
    for (int k = 0; k < K; ++k) lvl[k] = 0;
    for (int b = 0; b < B; ++b) {
        const uint16_t *xb = x + (size_t)b * K;
        int emax = -1;
        for (int k = 0; k < K; ++k) {
            uint16_t rm = rowmax[k] < 0x0400 ? (uint16_t)0x0400 : rowmax[k];
            float P = half_to_float(xb[k]) * half_to_float(rm);
            if (P != 0.0f && float_exp_field(P) > emax) emax = float_exp_field(P);
        }
        for (int k = 0; k < K; ++k) {
            uint16_t rm = rowmax[k] < 0x0400 ? (uint16_t)0x0400 : rowmax[k];
            float P = half_to_float(xb[k]) * half_to_float(rm);
            int level = 0;
            if (P != 0.0f) level = level_for_mantissa_bits(10 + guard_bits - (emax - float_exp_field(P)));
            if (level > lvl[k]) lvl[k] = (uint8_t)level;
        }
    }
    if (force_level >= 0)
        for (int k = 0; k < K; ++k) lvl[k] = (uint8_t)force_level;
    return 0;
}

/* y[b][n] = sum_k x[b][k] * W~[k][n] in binary64, ascending k; W~ = row k read at lvl[k].
 * y: [B][N]; lvl_out: [K] or NULL; abs_sum: [B][N] or NULL, sum_k |x[b][k] * W~[k][n]| (the scale
 * an accumulation error is measured against). */
int akwo_gemv(int B, int K, int N, const uint8_t *hi, const uint8_t *mid, const uint8_t *lo, const uint16_t *rowmax,
              const uint16_t *x, int guard_bits, int force_level, double *y, uint8_t *lvl_out, double *abs_sum)
{
    if (!shape_ok(K, N) || B < 1) return -1;
    uint8_t *lvl = (uint8_t *)malloc((size_t)K);
    if (!lvl) return -2;
    akwo_levels(B, K, x, rowmax, guard_bits, force_level, lvl);
    if (lvl_out) memcpy(lvl_out, lvl, (size_t)K);
    for (int b = 0; b < B; ++b)
        for (int n = 0; n < N; ++n) {
            double acc = 0.0, sa = 0.0;
            for (int k = 0; k < K; ++k) {
                double w = half_to_double(read_at_level(load_w(N, hi, mid, lo, k, n), lvl[k]));
                double t = half_to_double(x[(size_t)b * K + k]) * w;
                acc += t;
                sa += fabs(t);
            }
            y[(size_t)b * N + n] = acc;
            if (abs_sum) abs_sum[(size_t)b * N + n] = sa;
        }
    free(lvl);
    return 0;
}

double akwo_half_to_double(uint16_t h) { return half_to_double(h); }
uint16_t akwo_read_at_level(uint16_t h, int level) { return read_at_level(h, level); }
