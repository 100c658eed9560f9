// V side of decode attention as device functions: Rule 2 per element, fetch per token row, softmax
// weights, O = S V~.
// "Quantization of V-Cache": with O_est known, every addend s_t * v_td is aligned to the precision of the
// result (Rule 2); the bit width of the addend is the bit width V is read at.
#pragma once
#include "akv_common.h"

namespace akv {

// Byte-parallel form of Rule 2 for one token row.  With w_d = guard - 5 - Ehat_d and s = Ahat_t the
// mantissa bits element (t,d) needs are m = ev' + w_d + s (ev' = max(exponent field, 1)); the row is read
// at level >= 1 iff some m >= 3 and at level 2 iff some m >= 7.  Per byte: S = ev + B_d + (s + 64) with
// B_d = clamp(w_d + 61, 4, 132) reaches 128 exactly when ev + w_d + s reaches 3, and 132 exactly when it
// reaches 7: bit 7 of S and bit 7 of S - 4 are the two answers (no carry and no borrow: 4 <= S <= 227).
// The clamps only cut cases that are decided for every ev in 0..31 and s in -64..0.  ev' differs from ev
// only for ev = 0, which adds the row-independent test 1 + max_d w_d + s >= 3 (resp. 7).
__device__ __forceinline__ uint32_t clamp_byte(int v) { return (uint32_t)(v < 4 ? 4 : (v > 132 ? 132 : v)); }

// Per-lane constants of Rule 2 for the lane's 16 channels (lane -> channel slice 16 * (lane % 8))
struct VRule {
    uint32_t B[4];
    int ehat[16];   // only read by the variant that exports per-element needs
    int wmax;       // max over all 128 channels of w_d
    int force;      // -1, or the level every row is read at (then B = 4: no byte ever reaches bit 7)
};

// ehat: the 128 result exponents of the KV head (global memory or LDS)
__device__ __forceinline__ void v_rule_setup(const int* ehat, int guard_bits, int force_level, VRule& vr)
{
    const int cl = threadIdx.x & 7;
    int wmax = -100000;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        vr.B[i] = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int e = ehat[cl * 16 + i * 4 + k];
            vr.ehat[i * 4 + k] = e;
            const int w = guard_bits - 5 - e;
            wmax = w > wmax ? w : wmax;
            vr.B[i] |= clamp_byte(w + 61) << (8 * k);
        }
        if (force_level >= 0) vr.B[i] = 0x04040404u;
    }
    for (int o = 1; o < 8; o <<= 1) {
        const int other = __shfl_xor(wmax, o);
        wmax = other > wmax ? other : wmax;
    }
    vr.wmax = wmax;
    vr.force = force_level;
}

// OR over the 8 lanes of a row (lanes 8r .. 8r+7), result in all of them: two exchanges inside the quads,
// one with the mirrored lane of the 8-lane half row.
__device__ __forceinline__ uint32_t or_over_row(uint32_t v)
{
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, true);    // quad_perm [1,0,3,2]
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, true);    // quad_perm [2,3,0,1]
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xF, 0xF, true);   // row_half_mirror
    return v;
}

// HI bytes of the first NPRE batches of a wave, issued early by a caller that has idle time before the V side can
// start (they depend on nothing but the row range).  Rows at or past len are not fetched.
template <int KG, int NPRE>
__device__ __forceinline__ void v_prefetch_hi(const DecodeArgs& a, int b, int h, int t_first, int batch_stride, int len,
                                              u32x4_t (&hi)[NPRE][KG])
{
    const int lane = threadIdx.x & 63;
    const size_t bh = size_t(b) * a.s.Hkv + h;
    const __amdgpu_buffer_rsrc_t rs_hi = make_rsrc(a.v_hi + bh * a.s.Ncap * kD, uint32_t(len) * kD);
    const uint32_t voff = uint32_t(t_first) * kD + uint32_t(lane >> 3) * kD + uint32_t(lane & 7) * 16;
#pragma unroll
    for (int n = 0; n < NPRE; ++n)
#pragma unroll
        for (int gr = 0; gr < KG; ++gr) hi[n][gr] = buf_load_b128(rs_hi, voff + uint32_t(n * batch_stride + gr * 8) * kD);
}

// LDS of the shared mode of v_rows: the rows all waves of a workgroup assembled in one round, transposed -- line L
// holds one of the 128 values of a row (as fp16) for every row of the round, so that four consecutive rows of a line
// are one 8-byte read, the operand layout of the 16x16x16 matrix instruction -- and the weights of these rows, line
// g the high part and line G + g the low part of query head g's weight (two fp16 numbers whose sum carries 22 bits).
// Two buffers alternate by round.  Lines are kStride halves apart: 8-byte aligned, neighbouring lines two banks apart.
// Which channel a line holds: line_channel().
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
template <int G, int RB> struct VShare {
    static constexpr int kRows = kVWaves * RB;   // rows of a round
    static constexpr int kStride = kRows + 4;
    alignas(16) uint16_t vt[2][kD][kStride];
    alignas(16) uint16_t pt[2][16][kStride];
};
// assemble8_fill leaves channels (0,2), (1,3), (4,6), (5,7) of eight in its four words; the lane of channel slice cl
// stores half hf of word wi of its first eight channels in line 8 * (2 * wi + hf) + cl, of its second eight 64 lines on
__device__ __forceinline__ int line_channel(int line)
{
    const int c = (line & 63) >> 3, cl = line & 7, wi = c >> 1, hf = c & 1;
    return 16 * cl + 8 * (line >> 6) + (wi & 1) + 4 * (wi >> 1) + 2 * hf;
}
constexpr float kVWeightScale = 16384.0f;   // weights are at most 1: scaled by 2^14 their fp16 parts reach down to 2^-38
// workgroup barrier that waits for this wave's LDS traffic only: the loads from memory that are in flight stay in flight
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// One wave walks token rows of (b, h) in batches of 8*KG rows (KG groups of 8 rows; lane -> row lane/8 of the
// group and the 16-channel slice lane%8): batch i covers rows t_first + i*batch_stride .. + 8*KG - 1,
// i < nbatches.  Three stages per batch, software-pipelined over DL + 1 named buffers:
//   L  issue the HI loads and the logit load (lane j < 8*KG*G holds the logit of row j / G of the batch for query
//      head j % G: one load for all heads);
//   D  softmax weight and score exponent once per (row, head), in that lane, handed to the 8 lanes of the row by lane
//      permutes;
//      Rule 2 on the HI bytes; MID / LO loads of the rows that need them (the others are issued out of
//      range: nothing is fetched);
//   F  assemble the fp16 values, multiply-adds.
// Round i runs D(i+1), L(i+DL), F(i): every load has at least a whole round of arithmetic to arrive; a kernel
// with few waves per SIMD raises DL to keep enough bytes in flight.
// The descriptors end at row len, so rows at or past len read as zero without any per-lane test; their weight
// is forced to zero.  acc accumulates sum_t p_t * v~_td per lane (to be reduced over the 8 row lanes, then
// over waves, by the caller); z accumulates sum_t p_t per lane (to be summed over all 64 lanes).
// NPRE > 0: pre holds the HI bytes of batches 0 .. NPRE-1 (v_prefetch_hi) if pre_ok.
// lds_lg / lds_stride: the logits in LDS (query head g at lds_lg + g * lds_stride, token t at index t), or NULL: a.logits.
// NT: the HI bytes are read with the non-temporal hint (measured: it pays in the token-split V kernel, where the logits
// and the chunk partials of other workgroups share the caches, and costs in the head-per-workgroup kernel); the MID
// and LO bytes always are (it pays in both).
// SHARED, sh: the shared mode for groups of query heads (the token-split V kernel).  Every wave of the workgroup still
// fetches, tests and assembles its own rows, once, but leaves them in LDS (transposed) with their weights; after a
// barrier the sum over the rows of the round, for all query heads at once, is a matrix product on the matrix cores:
// D[m][line] += sum_rows W[m][row] * V[row][line], wave w taking lines 32 w .. 32 w + 31.  acc then holds the wave's two
// 16x16 result tiles (four words each: rows 4 * (lane / 16) .. + 3 of W, line 16 * (2 w + tile) + lane % 16), scaled by
// kVWeightScale.  A lane holds 8 sums instead of 16 * G, the multiply-adds leave the vector ALU.  All waves of the
// workgroup must call with the same nbatches.
template <int G, int KG, bool DEBUG, int NPRE, int DL = 2, bool NT = false, bool SHARED = false>
__device__ __forceinline__ void v_rows(const DecodeArgs& a, int b, int h, int t_first, int batch_stride, int nbatches,
                                       int len, const VRule& vr, const float (&Mg)[G], float (&acc)[SHARED ? 1 : G][SHARED ? 8 : 16],
                                       float (&z)[G], const u32x4_t (&pre)[NPRE > 0 ? NPRE : 1][KG], bool pre_ok,
                                       const float* lds_lg = nullptr, int lds_stride = 0, VShare<G, 8 * KG>* sh = nullptr)
{
    constexpr int RB = 8 * KG;
    static_assert(!SHARED || (G >= 4 && 2 * G <= 16 && kVWaves * 32 == kD && KG <= 2), "shared mode: high and low parts of all heads are the 16 rows of W; four waves share the 128 lines");
    const int wave = threadIdx.x >> 6;
    // wave-uniform by contract: scalar registers, scalar loop control
    nbatches = __builtin_amdgcn_readfirstlane(nbatches);
    t_first = __builtin_amdgcn_readfirstlane(t_first);
    if (nbatches <= 0) return;
    const int lane = threadIdx.x & 63;
    const int r = lane >> 3, cl = lane & 7;
    // lane j < RB * G computes the score of row j / G of the batch for query head j % G: every (row, head) pair once
    static_assert(RB * G <= 64 && (G & (G - 1)) == 0, "one lane per (row of the batch, query head)");
    const int jrow = lane / G, jg = lane % G;
    const bool jlane = lane < RB * G;
    const int Hkv = a.s.Hkv, Hq = a.s.Hq, Ncap = a.s.Ncap;
    const size_t bh = size_t(b) * Hkv + h;

    // the logits of the G query heads of the group lie Ncap floats apart: one descriptor over all of them
    const __amdgpu_buffer_rsrc_t rs_lg = make_rsrc(a.logits + (size_t(b) * Hq + size_t(h) * G) * Ncap, uint32_t(G) * uint32_t(Ncap) * 4u);
    const __amdgpu_buffer_rsrc_t rs_hi = make_rsrc(a.v_hi + bh * Ncap * kD, uint32_t(len) * kD);
    const __amdgpu_buffer_rsrc_t rs_mid = make_rsrc(a.v_mid + bh * Ncap * (kD / 2), uint32_t(len) * (kD / 2));
    const __amdgpu_buffer_rsrc_t rs_lo = make_rsrc(a.v_lo + bh * Ncap * (kD / 2), uint32_t(len) * (kD / 2));
    const uint32_t voff_hi = uint32_t(r) * kD + uint32_t(cl) * 16;
    const uint32_t voff_nib = uint32_t(r) * (kD / 2) + uint32_t(cl) * 8;
    const uint32_t voff_lg = (uint32_t(jg) * uint32_t(Ncap) + uint32_t(jrow)) * 4u;
    int src[KG];                                   // byte address of the first score lane of row gr*8 + r, for the lane permutes
#pragma unroll
    for (int gr = 0; gr < KG; ++gr) src[gr] = (gr * 8 + r) * G * 4;
    float Mlane = Mg[0];                           // the global max of this lane's query head
#pragma unroll
    for (int g = 1; g < G; ++g) Mlane = jg == g ? Mg[g] : Mlane;
    float zl = 0.0f;                               // sum of this lane's weights (rows j / G of the batches, head j % G)
    unsigned st_rows[3] = {0u, 0u, 0u}, st_need[3] = {0u, 0u, 0u};   // DEBUG: this lane's counts for akv_stats

    struct Batch {
        u32x4_t hi[KG];
        float lg;
        u32x2_t mid[KG], lo[KG];
        float p[SHARED ? 1 : KG][SHARED ? 1 : G];
        float pj;   // shared mode: the weight this lane computed, kept until the round of its batch
        uint32_t fill[KG];
    };
    auto row0 = [&](int bt) { return t_first + bt * batch_stride; };
    // a batch past the wave's last one is issued out of range: nothing is fetched
    auto Lhi = [&](Batch& X, int bt) {
        const uint32_t base = bt < nbatches ? uint32_t(row0(bt)) * kD : kSkip;
#pragma unroll
        for (int gr = 0; gr < KG; ++gr) X.hi[gr] = NT ? buf_load_b128_nt(rs_hi, voff_hi + base + gr * 8 * kD) : buf_load_b128(rs_hi, voff_hi + base + gr * 8 * kD);
    };
    auto Llg = [&](Batch& X, int bt) {   // one load for all heads; rows at or past len and idle lanes ask out of range
        const bool on = bt < nbatches && jlane && row0(bt) + jrow < len;
        if (lds_lg) X.lg = on ? lds_lg[jg * lds_stride + row0(bt) + jrow] : 0.0f;   // uniform branch: the kernel keeps its logits in LDS
        else X.lg = bits_float(buf_load_b32(rs_lg, on ? voff_lg + uint32_t(row0(bt)) * 4u : kSkip));
    };
    auto D = [&](Batch& X, int bt) {
        uint32_t offm[KG], offl[KG];
#pragma unroll
        for (int gr = 0; gr < KG; ++gr) offm[gr] = offl[gr] = kSkip;
        if (bt < nbatches) {   // uniform; arithmetic only -- the loads below are issued in any case
            const int t0 = row0(bt);
            const int nvalid = min(len - t0, RB);       // rows of the batch inside the sequence (may be <= 0)
            const float x = score_x(X.lg, Mlane, a.c);
            int ahat = score_a(x);                      // then the maximum over the G heads of the row (adjacent lanes)
            const float pj = jlane && jrow < nvalid ? __builtin_amdgcn_exp2f(x) : 0.0f;
            zl += pj;
            X.pj = pj;
            if (G >= 2) ahat = max(ahat, __builtin_amdgcn_update_dpp(ahat, ahat, 0xB1, 0xF, 0xF, false));    // quad_perm [1,0,3,2]
            if (G >= 4) ahat = max(ahat, __builtin_amdgcn_update_dpp(ahat, ahat, 0x4E, 0xF, 0xF, false));    // quad_perm [2,3,0,1]
            if (G >= 8) ahat = max(ahat, __builtin_amdgcn_update_dpp(ahat, ahat, 0x141, 0xF, 0xF, false));   // row_half_mirror
            const uint32_t ssw = __builtin_amdgcn_perm(0u, uint32_t(ahat + 64), 0x00000000u);   // (Ahat + 64) in every byte
            uint32_t Fw;   // bit 7: the row-independent test for level >= 1 holds, bit 15: the one for level 2
            if (vr.force >= 0) Fw = vr.force == 2 ? 0x8080u : (vr.force == 1 ? 0x0080u : 0u);
            else Fw = (ahat + 1 + vr.wmax >= 3 ? 0x0080u : 0u) | (ahat + 1 + vr.wmax >= 7 ? 0x8000u : 0u);
#pragma unroll
            for (int gr = 0; gr < KG; ++gr) {
                const uint32_t ss = (uint32_t)__builtin_amdgcn_ds_bpermute(src[gr], (int)ssw);
                const uint32_t Fg = (uint32_t)__builtin_amdgcn_ds_bpermute(src[gr], (int)Fw);
                if (!SHARED) {
#pragma unroll
                    for (int g = 0; g < G; ++g)
                        X.p[SHARED ? 0 : gr][SHARED ? 0 : g] = bits_float((uint32_t)__builtin_amdgcn_ds_bpermute(src[gr] + 4 * g, (int)float_bits(pj)));
                }
                const uint32_t hw[4] = {X.hi[gr].x, X.hi[gr].y, X.hi[gr].z, X.hi[gr].w};
                uint32_t any1 = Fg, any2 = Fg >> 8;   // bit 15 of Fg implies bit 7: stray bits in any1 do no harm
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t evp = (hw[i] >> 2) & 0x1F1F1F1Fu;
                    const uint32_t S = evp + vr.B[i] + ss;
                    any1 |= S;
                    any2 |= S - 0x04040404u;
                }
                // bit 7 of a byte: level >= 1 needed; bit 6: level 2 needed (which implies the former)
                const uint32_t flags = or_over_row((any1 & 0x80808080u) | ((any2 >> 1) & 0x40404040u));
                const bool need1 = flags != 0, need2 = (flags & 0x40404040u) != 0;
                const uint32_t off = voff_nib + uint32_t(t0) * (kD / 2) + gr * 8 * (kD / 2);
                offm[gr] = need1 ? off : kSkip;
                offl[gr] = need2 ? off : kSkip;
                X.fill[gr] = need2 ? 0u : (need1 ? 0x08080808u : 0x80808080u);

                if (DEBUG) {
                    const int t = t0 + gr * 8 + r;
                    if (t < len) {
                        const int applied = need2 ? 2 : (need1 ? 1 : 0);
                        if (a.dbg.appliedV && cl == 0) a.dbg.appliedV[bh * Ncap + t] = (uint8_t)applied;
                        if (cl == 0) {
                            st_rows[0] += applied == 0;
                            st_rows[1] += applied == 1;
                            st_rows[2] += applied == 2;
                        }
                        if (a.dbg.needV || a.stats) {
                            const int ah = int(ss & 0xFFu) - 64;
                            uint32_t nv[4];
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                nv[i] = 0;
#pragma unroll
                                for (int k = 0; k < 4; ++k) {
                                    int ev = (int)((hw[i] >> (8 * k + 2)) & 31u);
                                    ev = ev < 1 ? 1 : ev;
                                    int need = level_for_mantissa_bits(10 + a.guard_bits - (vr.ehat[i * 4 + k] - (ah + ev - 15)));
                                    if (a.force_level >= 0) need = a.force_level;
                                    nv[i] |= (uint32_t)need << (8 * k);
                                    st_need[1] += need == 1;
                                    st_need[2] += need == 2;
                                }
                            }
                            st_need[0] += 16;   // all of the lane's elements; those at levels 1 and 2 are taken off at the end
                            if (a.dbg.needV)
                                *reinterpret_cast<uint4*>(a.dbg.needV + (bh * Ncap + t) * kD + cl * 16) =
                                    make_uint4(nv[0], nv[1], nv[2], nv[3]);
                        }
                    }
                }
            }
        }
#pragma unroll
        for (int gr = 0; gr < KG; ++gr) {
            X.mid[gr] = buf_load_b64_nt(rs_mid, offm[gr]);
            X.lo[gr] = buf_load_b64_nt(rs_lo, offl[gr]);
        }
    };
    auto F = [&](const Batch& X, int bt) {
        if (bt >= nbatches) return;
#pragma unroll
        for (int gr = 0; gr < KG; ++gr) {
            uint32_t pa[4], pb[4];
            assemble8_fill(X.hi[gr].x, X.hi[gr].y, X.mid[gr].x, X.lo[gr].x, X.fill[gr], pa);   // channels 0..7 of the slice
            assemble8_fill(X.hi[gr].z, X.hi[gr].w, X.mid[gr].y, X.lo[gr].y, X.fill[gr], pb);   // channels 8..15
            const float v[16] = {lo_half(pa[0]), lo_half(pa[1]), hi_half(pa[0]), hi_half(pa[1]),
                                 lo_half(pa[2]), lo_half(pa[3]), hi_half(pa[2]), hi_half(pa[3]),
                                 lo_half(pb[0]), lo_half(pb[1]), hi_half(pb[0]), hi_half(pb[1]),
                                 lo_half(pb[2]), lo_half(pb[3]), hi_half(pb[2]), hi_half(pb[3])};
#pragma unroll
            for (int g = 0; g < (SHARED ? 1 : G); ++g)
#pragma unroll
                for (int i = 0; i < (SHARED ? 8 : 16); ++i) acc[g][i] = fmaf(X.p[SHARED ? 0 : gr][SHARED ? 0 : g], v[i], acc[g][i]);
        }
    };

    // shared mode: A leaves the wave's rows of batch bt, transposed, and their weights in the round's buffer; Fs is the
    // wave's share of the matrix product over the rows of the round
    auto A = [&](const Batch& X, int bt) {
        const int buf = bt & 1;
        uint32_t pa[KG][4], pb[KG][4];
#pragma unroll
        for (int gr = 0; gr < KG; ++gr) {
            assemble8_fill(X.hi[gr].x, X.hi[gr].y, X.mid[gr].x, X.lo[gr].x, X.fill[gr], pa[gr]);
            assemble8_fill(X.hi[gr].z, X.hi[gr].w, X.mid[gr].y, X.lo[gr].y, X.fill[gr], pb[gr]);
        }
        // the order of the rows inside a round is free (the weights follow it): the lane's two rows, 8 apart in the
        // batch, are neighbours in the buffer, so that one 32-bit store lays down both
        const int row = wave * RB + KG * r;
#pragma unroll
        for (int wi = 0; wi < 4; ++wi) {
            if (KG == 2) {
                *reinterpret_cast<uint32_t*>(&sh->vt[buf][8 * (2 * wi) + cl][row]) = __builtin_amdgcn_perm(pa[KG - 1][wi], pa[0][wi], 0x05040100u);
                *reinterpret_cast<uint32_t*>(&sh->vt[buf][8 * (2 * wi + 1) + cl][row]) = __builtin_amdgcn_perm(pa[KG - 1][wi], pa[0][wi], 0x07060302u);
                *reinterpret_cast<uint32_t*>(&sh->vt[buf][64 + 8 * (2 * wi) + cl][row]) = __builtin_amdgcn_perm(pb[KG - 1][wi], pb[0][wi], 0x05040100u);
                *reinterpret_cast<uint32_t*>(&sh->vt[buf][64 + 8 * (2 * wi + 1) + cl][row]) = __builtin_amdgcn_perm(pb[KG - 1][wi], pb[0][wi], 0x07060302u);
            } else {
                sh->vt[buf][8 * (2 * wi) + cl][row] = (uint16_t)pa[0][wi];
                sh->vt[buf][8 * (2 * wi + 1) + cl][row] = (uint16_t)(pa[0][wi] >> 16);
                sh->vt[buf][64 + 8 * (2 * wi) + cl][row] = (uint16_t)pb[0][wi];
                sh->vt[buf][64 + 8 * (2 * wi + 1) + cl][row] = (uint16_t)(pb[0][wi] >> 16);
            }
        }
        if (jlane) {
            const float ws = X.pj * kVWeightScale;
            const _Float16 whi = (_Float16)ws;
            const _Float16 wlo = (_Float16)(ws - (float)whi);
            const int wrow = wave * RB + KG * (jrow & 7) + (jrow >> 3);
            sh->pt[buf][jg][wrow] = __builtin_bit_cast(uint16_t, whi);
            sh->pt[buf][G + jg][wrow] = __builtin_bit_cast(uint16_t, wlo);
        }
    };
    f32x4_t d0 = {0.0f, 0.0f, 0.0f, 0.0f}, d1 = {0.0f, 0.0f, 0.0f, 0.0f};   // the wave's two result tiles
    auto Fs = [&](int bt) {
        const int buf = bt & 1;
        const int n = lane & 15, kq = 4 * (lane >> 4);
#pragma unroll
        for (int kb = 0; kb < (kVWaves * RB) / 16; ++kb) {
            const half4_t w4 = *reinterpret_cast<const half4_t*>(&sh->pt[buf][n][kb * 16 + kq]);
            const half4_t v0 = *reinterpret_cast<const half4_t*>(&sh->vt[buf][32 * wave + n][kb * 16 + kq]);
            const half4_t v1 = *reinterpret_cast<const half4_t*>(&sh->vt[buf][32 * wave + 16 + n][kb * 16 + kq]);
            d0 = __builtin_amdgcn_mfma_f32_16x16x16f16(w4, v0, d0, 0, 0, 0);
            d1 = __builtin_amdgcn_mfma_f32_16x16x16f16(w4, v1, d1, 0, 0, 0);
        }
    };
    if constexpr (SHARED && 2 * G < 16) {   // the rows of W no head uses stay zero in both buffers (ordered before the first read by the first barrier)
        for (int idx = threadIdx.x; idx < 2 * (16 - 2 * G) * VShare<G, RB>::kStride; idx += 64 * kVWaves) {
            const int bf = idx / ((16 - 2 * G) * VShare<G, RB>::kStride), rest = idx % ((16 - 2 * G) * VShare<G, RB>::kStride);
            sh->pt[bf][2 * G + rest / VShare<G, RB>::kStride][rest % VShare<G, RB>::kStride] = 0;
        }
    }

    // R = DL + 1 named buffers: round i runs D(i + 1), L(i + DL), F(i); the buffer L fills is the one F emptied in
    // the round before.  The loop is unrolled R times so that every buffer index is a constant.  Loads come back in
    // the order they were issued, so the wait of F(i) for its MID / LO bytes (asked for by D(i), one round earlier) is
    // also a wait for every load issued before them: D issues ahead of L in a round, so that this never includes the HI
    // bytes L asked for in that round.
    constexpr int R = DL + 1;
    static_assert(DL >= 2 && NPRE <= DL, "the HI loads run at least two batches ahead");
    Batch ring[R];
#pragma unroll
    for (int k = 0; k < DL; ++k) {
        if (k < NPRE) {
#pragma unroll
            for (int gr = 0; gr < KG; ++gr) ring[k].hi[gr] = pre[k < NPRE ? k : 0][gr];
            if (!pre_ok) Lhi(ring[k], k);
        } else {
            Lhi(ring[k], k);
        }
        Llg(ring[k], k);
    }
    D(ring[0], 0);
#pragma unroll 1
    for (int i = 0; i < nbatches; i += R) {   // rounds past the last batch issue nothing and compute nothing
#pragma unroll
        for (int k = 0; k < R; ++k) {
            D(ring[(k + 1) % R], i + k + 1);
            Lhi(ring[(k + DL) % R], i + k + DL);
            Llg(ring[(k + DL) % R], i + k + DL);
            if (SHARED) {
                if (i + k < nbatches) {   // the same for every wave of the workgroup
                    A(ring[k], i + k);
                    lds_barrier();
                    Fs(i + k);
                }
            } else {
                F(ring[k], i + k);
            }
        }
    }
#pragma unroll
    for (int g = 0; g < G; ++g) z[g] += jg == g ? zl : 0.0f;
    if (SHARED) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            acc[0][i] = d0[i];
            acc[0][SHARED ? 4 + i : 0] = d1[i];
        }
    }
    if (DEBUG && a.stats) {   // uniform; one set of atomics per wave
        st_need[0] -= st_need[1] + st_need[2];
        unsigned v6[6] = {st_rows[0], st_rows[1], st_rows[2], st_need[0], st_need[1], st_need[2]};
#pragma unroll
        for (int i = 0; i < 6; ++i)
            for (int o = 1; o < 64; o <<= 1) v6[i] += __shfl_xor(v6[i], o);
        if (lane == 0) {
#pragma unroll
            for (int i = 0; i < 3; ++i) {
                atomicAdd(reinterpret_cast<unsigned long long*>(&a.stats->v_row_elems[i]), (unsigned long long)v6[i] * kD);
                atomicAdd(reinterpret_cast<unsigned long long*>(&a.stats->v_need_elems[i]), (unsigned long long)v6[3 + i]);
            }
        }
    }
}

// sum acc over the 8 row lanes of a wave (lanes with the same lane % 8) and z over all lanes; afterwards
// lanes 0..7 hold the wave's totals for their channel slices and every lane holds the wave's z
template <int G>
__device__ __forceinline__ void v_reduce_rows(float (&acc)[G][16], float (&z)[G])
{
#pragma unroll
    for (int g = 0; g < G; ++g) {
        for (int o = 1; o < 64; o <<= 1) z[g] += __shfl_xor(z[g], o);
        for (int o = 8; o < 64; o <<= 1) {
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[g][i] += __shfl_xor(acc[g][i], o);
        }
    }
}

// write out[b][h*G + g][:] = o / zsum for channel d (or zero for an empty sequence)
__device__ __forceinline__ void store_out(const DecodeArgs& a, size_t hq, int d, float res)
{
    if (a.out_dtype == 0) reinterpret_cast<float*>(a.out)[hq * kD + d] = res;
    else reinterpret_cast<_Float16*>(a.out)[hq * kD + d] = (_Float16)res;
}

}  // namespace akv
