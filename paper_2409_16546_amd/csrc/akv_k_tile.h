// K side of decode attention as device functions: Rule 1 level per K column, and the streaming q.K~ pass
// over one tile of tokens.
// "Quantization of K-Cache": from q and K_colmax estimate the magnitude of the 128 addends of one logit,
// align them to the coarsest one (Rule 1), read each column of K at the bit width its addend needs.
#pragma once
#include "akv_common.h"

namespace akv {

// LDS of the K side of one (sequence, KV head)
template <int G>
struct KShared {
    float q[G][kD];
    int emax[G];
    uint64_t need_mid[2], need_lo[2];   // bit d%64 of word d/64: column d is read at level >= 1 / = 2
    float knew[kD];                     // fused append: the new token's K row as it will be read at the column levels
    float new_logit[G];                 // fused append: q . knew, accumulated in channel order
};

// Rule 1 for the 128 columns of (b, h).  Called by every thread of a workgroup of at least 128 threads
// (contains barriers); afterwards ks holds q as fp32 and the level masks.
// k_new_bits: fp16 bits of channel tid of a token that is being appended in the same kernel (fused append),
// else -1: K_colmax then counts that token, and the token's row, read at the column levels, is left in
// ks.knew for new_token_logit().  Returns the K_colmax of channel tid (tid < 128) that the levels used.
template <int G>
__device__ __forceinline__ uint32_t k_levels(const DecodeArgs& a, int b, int h, KShared<G>& ks, bool export_levels,
                                             int k_new_bits = -1)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const size_t bh = size_t(b) * a.s.Hkv + h;
    if (tid < G) ks.emax[tid] = -1;
    __syncthreads();
    float P[G];
    uint32_t colmax_used = 0;
    if (tid < kD) {
        uint32_t cm = a.colmax[bh * kD + tid];
        if (k_new_bits >= 0) cm = max(cm, uint32_t(k_new_bits) & 0x7FFFu);
        colmax_used = cm;
        cm = cm < 0x0400u ? 0x0400u : cm;               // below the smallest normal: its places are 2^-14's
        const float cmf = half_bits_to_float(cm);
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float qf = half_bits_to_float(a.q[(size_t(b) * a.s.Hq + size_t(h) * G + g) * kD + tid]);
            ks.q[g][tid] = qf;
            P[g] = qf * cmf;                             // exact: 11-bit x 11-bit significands
            if (P[g] != 0.0f) atomicMax(&ks.emax[g], float_exp_field(P[g]));
        }
    }
    __syncthreads();
    if (tid < kD) {   // waves 0 and 1: channel tid
        int lv = 0;
#pragma unroll
        for (int g = 0; g < G; ++g) {
            if (P[g] != 0.0f) {
                const int l = level_for_mantissa_bits(10 + a.guard_bits - (ks.emax[g] - float_exp_field(P[g])));
                lv = l > lv ? l : lv;
            }
        }
        if (a.force_level >= 0) lv = a.force_level;
        const uint64_t b1 = __ballot(lv >= 1), b2 = __ballot(lv >= 2);
        if (lane == 0) {
            ks.need_mid[wave] = b1;
            ks.need_lo[wave] = b2;
        }
        if (a.dbg.lvlK && export_levels) a.dbg.lvlK[bh * kD + tid] = (uint8_t)lv;
        if (k_new_bits >= 0) {   // "Dynamic Quantization": bits that are not read are filled with 100...
            const uint32_t kb = uint32_t(k_new_bits);
            ks.knew[tid] = half_bits_to_float(lv == 2 ? kb : (lv == 1 ? ((kb & 0xFFF0u) | 0x0008u) : ((kb & 0xFF00u) | 0x0080u)));
        }
    }
    __syncthreads();
    return colmax_used;
}

// Fused append: the logit of the token that is being appended, from ks.knew, with the same arithmetic as a
// tile lane (fp32, channels ascending).  One thread per query head of the group.
template <int G>
__device__ __forceinline__ float new_token_logit(const KShared<G>& ks, int g)
{
    float acc = 0.0f;
    for (int d0 = 0; d0 < kD; d0 += 16) {   // operands fetched 16 at a time, the additions stay in channel order
        float qv[16], kv[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            qv[i] = ks.q[g][d0 + i];
            kv[i] = ks.knew[d0 + i];
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) acc = fmaf(qv[i], kv[i], acc);
    }
    return acc;
}

__device__ __forceinline__ uint64_t uniform64(uint64_t v)
{   // readfirstlane returns a signed int: widen through uint32_t
    const uint32_t lo32 = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
    const uint32_t hi32 = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(v >> 32));
    return (uint64_t(hi32) << 32) | uint64_t(lo32);
}

// One wave, one tile of 64*TPL tokens of (b, h) starting at 256-token block blk0: lane -> TPL consecutive
// tokens of one block (TPL = 4: the wave reads one contiguous 256-B run of K_hi per channel; TPL = 8: two
// runs, one per block).  Channels are processed U at a time.
// If the column's level asks for it the matching runs of K_mid / K_lo are read as well.  Every byte is used
// by exactly one lane, so nothing is staged through LDS.  The logit of a token is accumulated in fp32 over
// channels in ascending order (one lane, no reduction).  Logits go to a.logits with cache policy `aux`
// (kAuxSc1 when another workgroup of the same kernel will read them); the maximum over the tile's valid
// tokens is returned for every query head of the group (same value in all lanes).
template <int G, int TPL, int U>
__device__ __forceinline__ void k_tile(const DecodeArgs& a, int b, int h, int blk0, int len, const KShared<G>& ks,
                                       int aux, float (&tile_max)[G])
{
    static_assert(TPL == 4 || TPL == 8, "tokens per lane");
    static_assert(U == 4 || U == 8, "channels per group");
    constexpr int kLanesPerBlock = kTB / TPL;
    const int lane = threadIdx.x & 63;
    const int Hkv = a.s.Hkv, Hq = a.s.Hq, Ncap = a.s.Ncap, NB = Ncap / kTB;
    const size_t bh = size_t(b) * Hkv + h;

    const int blk = blk0 + lane / kLanesPerBlock;
    const bool live = blk < NB;                          // Ncap may end inside the tile
    const int blk_ld = live ? blk : NB - 1;              // such lanes re-read the last block and store nothing
    const int j0 = (lane % kLanesPerBlock) * TPL;
    const uint32_t off_hi = uint32_t(blk_ld) * kD * kTB + j0;
    const uint32_t off_nib = uint32_t(blk_ld) * kD * (kTB / 2) + j0 / 2;

    float acc[G][TPL];
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
        for (int i = 0; i < TPL; ++i) acc[g][i] = 0.0f;

    // the level masks live in scalar registers for the whole loop
    const uint64_t nm0 = uniform64(ks.need_mid[0]), nm1 = uniform64(ks.need_mid[1]);
    const uint64_t nl0 = uniform64(ks.need_lo[0]), nl1 = uniform64(ks.need_lo[1]);

    struct Group {
        uint32_t h0[U], h1[U];   // HI bytes of tokens 0..3 / 4..7 (h1 unused for TPL = 4)
        uint32_t m[U], l[U];     // MID / LO nibbles, token 2i in the low nibble of byte i
    };
    // bits of the U channels starting at d0 (d0 % U == 0, so a group never straddles the two words)
    auto bits_at = [&](uint64_t w0, uint64_t w1, int d0) -> uint32_t {
        return d0 < kD ? (uint32_t)((d0 < 64 ? w0 : w1) >> (d0 & 63)) & ((1u << U) - 1) : 0u;
    };
    // A plane that a column does not need is read through a descriptor of size zero: the range check then
    // answers every lane with zero and nothing is fetched.  The choice is scalar (the level is per column),
    // the per-lane offset is the same register for every load, the channel goes into the scalar offset.
    const uint32_t slab = uint32_t(Ncap) * (kD / 2);
    auto issue = [&](Group& gr, int d0) {
        const uint32_t bm = bits_at(nm0, nm1, d0), bl = bits_at(nl0, nl1, d0);
        const __amdgpu_buffer_rsrc_t rh = make_rsrc(a.k_hi + bh * Ncap * kD, d0 < kD ? 2 * slab : 0u);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const __amdgpu_buffer_rsrc_t rm = make_rsrc(a.k_mid + bh * Ncap * (kD / 2), ((bm >> u) & 1u) ? slab : 0u);
            const __amdgpu_buffer_rsrc_t rl = make_rsrc(a.k_lo + bh * Ncap * (kD / 2), ((bl >> u) & 1u) ? slab : 0u);
            if constexpr (TPL == 8) {
                const u32x2_t hh = __builtin_amdgcn_raw_buffer_load_b64(rh, off_hi + u * kTB, d0 * kTB, 0);
                gr.h0[u] = hh.x;
                gr.h1[u] = hh.y;
                gr.m[u] = __builtin_amdgcn_raw_buffer_load_b32(rm, off_nib + u * (kTB / 2), d0 * (kTB / 2), 0);
                gr.l[u] = __builtin_amdgcn_raw_buffer_load_b32(rl, off_nib + u * (kTB / 2), d0 * (kTB / 2), 0);
            } else {
                gr.h0[u] = __builtin_amdgcn_raw_buffer_load_b32(rh, off_hi + u * kTB, d0 * kTB, 0);
                gr.m[u] = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rm, off_nib + u * (kTB / 2), d0 * (kTB / 2), 0);
                gr.l[u] = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rl, off_nib + u * (kTB / 2), d0 * (kTB / 2), 0);
            }
        }
    };
    auto compute = [&](const Group& gr, int d0) {
        const uint32_t bm = bits_at(nm0, nm1, d0), bl = bits_at(nl0, nl1, d0);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            uint32_t ev, od;   // low bytes of tokens 0,2,4,6 / 1,3,5,7
            if ((bl >> u) & 1u) {   // all 16 bits read (uniform branch)
                ev = ((gr.m[u] << 4) & 0xF0F0F0F0u) | (gr.l[u] & 0x0F0F0F0Fu);
                od = (gr.m[u] & 0xF0F0F0F0u) | ((gr.l[u] >> 4) & 0x0F0F0F0Fu);
            } else {                // 12 bits (MID read, fill 1000) or 8 bits (MID word is zero, fill 1000 0000)
                const uint32_t fill = ((bm >> u) & 1u) ? 0x08080808u : 0x80808080u;
                ev = ((gr.m[u] << 4) & 0xF0F0F0F0u) | fill;
                od = (gr.m[u] & 0xF0F0F0F0u) | fill;
            }
            float k[TPL];
            const uint32_t p0 = __builtin_amdgcn_perm(gr.h0[u], ev, 0x06010400u);   // tokens (0,2)
            const uint32_t p1 = __builtin_amdgcn_perm(gr.h0[u], od, 0x07010500u);   // tokens (1,3)
            k[0] = lo_half(p0); k[2] = hi_half(p0); k[1] = lo_half(p1); k[3] = hi_half(p1);
            if constexpr (TPL == 8) {
                const uint32_t p2 = __builtin_amdgcn_perm(gr.h1[u], ev, 0x06030402u);   // tokens (4,6)
                const uint32_t p3 = __builtin_amdgcn_perm(gr.h1[u], od, 0x07030502u);   // tokens (5,7)
                k[4] = lo_half(p2); k[6] = hi_half(p2); k[5] = lo_half(p3); k[7] = hi_half(p3);
            }
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const float qd = ks.q[g][d0 + u];
                // q*k is exact in fp32, so the fused form rounds exactly like multiply-then-add
#pragma unroll
                for (int i = 0; i < TPL; ++i) acc[g][i] = fmaf(qd, k[i], acc[g][i]);
            }
        }
    };
    // three groups rotate by name: two are in flight while one is consumed (48 loads outstanding at most,
    // below the 6-bit counter of outstanding vector-memory operations)
    Group A, B, C;
    issue(A, 0);
    issue(B, U);
#pragma unroll 1
    for (int d0 = 0; d0 < kD; d0 += 3 * U) {
        issue(C, d0 + 2 * U);
        compute(A, d0);
        issue(A, d0 + 3 * U);
        if (d0 + U < kD) compute(B, d0 + U);   // kD is not a multiple of 3 * U: the last round is partial
        issue(B, d0 + 4 * U);
        if (d0 + 2 * U < kD) compute(C, d0 + 2 * U);
    }

    // ---- logits out, tile maxima -----------------------------------------------------------------
    const int t0 = blk * kTB + j0;
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const size_t hq = size_t(b) * Hq + size_t(h) * G + g;
        const __amdgpu_buffer_rsrc_t rs_lg = make_rsrc(a.logits + hq * Ncap, uint32_t(Ncap) * 4u);
#pragma unroll
        for (int i = 0; i < TPL; i += 4) {
            u32x4_t w;
            w.x = float_bits(acc[g][i]); w.y = float_bits(acc[g][i + 1]);
            w.z = float_bits(acc[g][i + 2]); w.w = float_bits(acc[g][i + 3]);
            const uint32_t off = live ? uint32_t(t0 + i) * 4u : kSkip;   // out of range: the store is dropped
            if (aux) __builtin_amdgcn_raw_buffer_store_b128(w, rs_lg, off, 0, kAuxSc1);
            else __builtin_amdgcn_raw_buffer_store_b128(w, rs_lg, off, 0, 0);
        }
        float m = -INFINITY;
#pragma unroll
        for (int i = 0; i < TPL; ++i)
            if (live && t0 + i < len) m = fmaxf(m, acc[g][i]);
        tile_max[g] = wave_max(m);
    }
}

}  // namespace akv
