// V side of decode attention as device functions: Rule 2 per element, fetch per token row, softmax
// weights, O = S V~.
// "Quantization of V-Cache": with O_est known, every addend s_t * v_td is aligned to the precision of the
// result (Rule 2); the bit width of the addend is the bit width V is read at.
#pragma once
#include "akv_common.h"

namespace akv {

// Byte-parallel form of Rule 2 for one token row.  With w_d = guard - 5 - Ehat_d and s = Ahat_t the
// mantissa bits element (t,d) needs are m = ev' + w_d + s (ev' = max(exponent field, 1)); the row is read
// at level >= 1 iff some m >= 3 and at level 2 iff some m >= 7.  Per byte: ev + B + (s + 64) with
// B1_d = clamp(w_d + 61, 0, 128), B2_d = clamp(w_d + 57, 0, 128) sets bit 7 exactly when ev + w_d + s
// reaches 3 resp. 7 (no carry: the sum is at most 31 + 128 + 64); the clamps only cut cases that are
// decided for every ev in 0..31 and s in -64..0.  ev' differs from ev only for ev = 0, which adds the
// row-independent test 1 + max_d w_d + s >= 3 (resp. 7).
__device__ __forceinline__ uint32_t clamp_byte(int v) { return (uint32_t)(v < 0 ? 0 : (v > 128 ? 128 : v)); }

// Per-lane constants of Rule 2 for the lane's 16 channels (lane -> channel slice 16 * (lane % 8))
struct VRule {
    uint32_t B1[4], B2[4];
    int ehat[16];   // only read by the variant that exports per-element needs
    int wmax;       // max over all 128 channels of w_d
};

// ehat: the 128 result exponents of the KV head (global memory or LDS)
__device__ __forceinline__ void v_rule_setup(const int* ehat, int guard_bits, VRule& vr)
{
    const int cl = threadIdx.x & 7;
    int wmax = -100000;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        vr.B1[i] = 0;
        vr.B2[i] = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int e = ehat[cl * 16 + i * 4 + k];
            vr.ehat[i * 4 + k] = e;
            const int w = guard_bits - 5 - e;
            wmax = w > wmax ? w : wmax;
            vr.B1[i] |= clamp_byte(w + 61) << (8 * k);
            vr.B2[i] |= clamp_byte(w + 57) << (8 * k);
        }
    }
    for (int o = 1; o < 8; o <<= 1) {
        const int other = __shfl_xor(wmax, o);
        wmax = other > wmax ? other : wmax;
    }
    vr.wmax = wmax;
}

// One wave walks token rows of (b, h) in batches of 32 (4 groups of 8 rows; lane -> row lane/8 of the group
// and the 16-channel slice lane%8): batch i covers rows t_first + i*batch_stride .. +31, i < nbatches.  Per
// batch: decide the 32 rows from their HI bytes, issue the MID / LO loads of the rows that need them, issue
// the HI loads of the next batch, and only then do the multiply-adds, so that the dependent MID / LO fetch and
// the next HI fetch are both in flight behind the arithmetic.  Rows at or past len contribute nothing.
// acc / z accumulate sum_t p_t * v~_td and sum_t p_t per lane (to be reduced over the 8 row lanes, then over
// waves, by the caller).
template <int G, bool DEBUG>
__device__ __forceinline__ void v_rows(const DecodeArgs& a, int b, int h, int t_first, int batch_stride, int nbatches,
                                       int len, const VRule& vr, const float (&Mg)[G], float (&acc)[G][16],
                                       float (&z)[G])
{
    constexpr int kGroups = 4;   // row groups (of 8 rows) per batch
    const int lane = threadIdx.x & 63;
    const int r = lane >> 3, cl = lane & 7;
    const int Hkv = a.s.Hkv, Hq = a.s.Hq, Ncap = a.s.Ncap;
    const size_t bh = size_t(b) * Hkv + h;

    __amdgpu_buffer_rsrc_t rs_lg[G];
#pragma unroll
    for (int g = 0; g < G; ++g)
        rs_lg[g] = make_rsrc(a.logits + (size_t(b) * Hq + size_t(h) * G + g) * Ncap, uint32_t(Ncap) * 4u);
    const __amdgpu_buffer_rsrc_t rs_hi = make_rsrc(a.v_hi + bh * Ncap * kD, uint32_t(Ncap) * kD);
    const __amdgpu_buffer_rsrc_t rs_mid = make_rsrc(a.v_mid + bh * Ncap * (kD / 2), uint32_t(Ncap) * (kD / 2));
    const __amdgpu_buffer_rsrc_t rs_lo = make_rsrc(a.v_lo + bh * Ncap * (kD / 2), uint32_t(Ncap) * (kD / 2));

    u32x4_t hc[kGroups], hn[kGroups];       // HI bytes of the current / the next batch
    float lc[kGroups][G], ln[kGroups][G];   // logits of the current / the next batch
    auto load_batch = [&](int bt, u32x4_t (&hh)[kGroups], float (&ll)[kGroups][G]) {
#pragma unroll
        for (int gr = 0; gr < kGroups; ++gr) {
            const int t = t_first + bt * batch_stride + gr * 8 + r;
            const bool valid = t < len && bt < nbatches;   // past the wave's rows: nothing is fetched
            hh[gr] = buf_load_b128(rs_hi, valid ? uint32_t(t) * kD + cl * 16 : kSkip);
#pragma unroll
            for (int g = 0; g < G; ++g) ll[gr][g] = bits_float(buf_load_b32(rs_lg[g], valid ? uint32_t(t) * 4u : kSkip));
        }
    };
    load_batch(0, hc, lc);

#pragma unroll 1
    for (int bt = 0; bt < nbatches; ++bt) {
        float p[kGroups][G];
        u32x2_t mid[kGroups], lo[kGroups];
        uint32_t fill[kGroups];
        // decisions of the batch, then its MID / LO loads
#pragma unroll
        for (int gr = 0; gr < kGroups; ++gr) {
            const int t = t_first + bt * batch_stride + gr * 8 + r;
            const bool valid = t < len;
            int ahat = kAMin;
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const float x = score_x(lc[gr][g], Mg[g], a.c);
                const int ag = score_a(x);
                ahat = ag > ahat ? ag : ahat;
                p[gr][g] = valid ? __builtin_amdgcn_exp2f(x) : 0.0f;
            }
            const uint32_t ssplat = (uint32_t)(ahat + 64) * 0x01010101u;
            const uint32_t hw[4] = {hc[gr].x, hc[gr].y, hc[gr].z, hc[gr].w};
            uint32_t any1 = 0, any2 = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t evp = (hw[i] >> 2) & 0x1F1F1F1Fu;
                any1 |= evp + vr.B1[i] + ssplat;
                any2 |= evp + vr.B2[i] + ssplat;
            }
            const uint64_t b1 = __ballot((any1 & 0x80808080u) != 0), b2 = __ballot((any2 & 0x80808080u) != 0);
            const int sh = lane & 56;
            const bool need1 = ((b1 >> sh) & 0xFFu) != 0 || (ahat + 1 + vr.wmax >= 3);
            const bool need2 = ((b2 >> sh) & 0xFFu) != 0 || (ahat + 1 + vr.wmax >= 7);
            int applied = need2 ? 2 : (need1 ? 1 : 0);
            if (a.force_level >= 0) applied = a.force_level;
            const uint32_t off = uint32_t(t) * (kD / 2) + cl * 8;
            mid[gr] = buf_load_b64(rs_mid, (valid && applied >= 1) ? off : kSkip);
            lo[gr] = buf_load_b64(rs_lo, (valid && applied >= 2) ? off : kSkip);
            fill[gr] = fill_for_level(applied);

            if (DEBUG && valid) {
                if (a.dbg.appliedV && cl == 0) a.dbg.appliedV[bh * Ncap + t] = (uint8_t)applied;
                if (a.dbg.needV) {
                    uint32_t nv[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        nv[i] = 0;
#pragma unroll
                        for (int k = 0; k < 4; ++k) {
                            int ev = (int)((hw[i] >> (8 * k + 2)) & 31u);
                            ev = ev < 1 ? 1 : ev;
                            int need = level_for_mantissa_bits(10 + a.guard_bits - (vr.ehat[i * 4 + k] - (ahat + ev - 15)));
                            if (a.force_level >= 0) need = a.force_level;
                            nv[i] |= (uint32_t)need << (8 * k);
                        }
                    }
                    *reinterpret_cast<uint4*>(a.dbg.needV + (bh * Ncap + t) * kD + cl * 16) =
                        make_uint4(nv[0], nv[1], nv[2], nv[3]);
                }
            }
        }
        // HI bytes and logits of the next batch go in flight behind the MID / LO loads
        load_batch(bt + 1, hn, ln);
        // multiply-adds of the batch
#pragma unroll
        for (int gr = 0; gr < kGroups; ++gr) {
            uint32_t pa[4], pb[4];
            assemble8_fill(hc[gr].x, hc[gr].y, mid[gr].x, lo[gr].x, fill[gr], pa);   // channels 0..7 of the slice
            assemble8_fill(hc[gr].z, hc[gr].w, mid[gr].y, lo[gr].y, fill[gr], pb);   // channels 8..15
            const float v[16] = {lo_half(pa[0]), lo_half(pa[1]), hi_half(pa[0]), hi_half(pa[1]),
                                 lo_half(pa[2]), lo_half(pa[3]), hi_half(pa[2]), hi_half(pa[3]),
                                 lo_half(pb[0]), lo_half(pb[1]), hi_half(pb[0]), hi_half(pb[1]),
                                 lo_half(pb[2]), lo_half(pb[3]), hi_half(pb[2]), hi_half(pb[3])};
#pragma unroll
            for (int g = 0; g < G; ++g) {
                z[g] += p[gr][g];
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[g][i] = fmaf(p[gr][g], v[i], acc[g][i]);
            }
        }
#pragma unroll
        for (int gr = 0; gr < kGroups; ++gr) {
            hc[gr] = hn[gr];
#pragma unroll
            for (int g = 0; g < G; ++g) lc[gr][g] = ln[gr][g];
        }
    }
}

// sum acc / z over the 8 row lanes of a wave (lanes with the same lane % 8); afterwards lanes 0..7 hold the
// wave's totals for their channel slices
template <int G>
__device__ __forceinline__ void v_reduce_rows(float (&acc)[G][16], float (&z)[G])
{
#pragma unroll
    for (int g = 0; g < G; ++g)
        for (int o = 8; o < 64; o <<= 1) {
            z[g] += __shfl_xor(z[g], o);
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[g][i] += __shfl_xor(acc[g][i], o);
        }
}

// write out[b][h*G + g][:] = o / zsum for channel d (or zero for an empty sequence)
__device__ __forceinline__ void store_out(const DecodeArgs& a, size_t hq, int d, float res)
{
    if (a.out_dtype == 0) reinterpret_cast<float*>(a.out)[hq * kD + d] = res;
    else reinterpret_cast<_Float16*>(a.out)[hq * kD + d] = (_Float16)res;
}

}  // namespace akv
