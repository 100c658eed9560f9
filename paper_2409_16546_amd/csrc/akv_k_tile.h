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
    int emax[2][G];                     // largest addend exponent per query head, of the columns of wave 0 / wave 1
    uint64_t need_mid[2], need_lo[2];   // bit d%64 of word d/64: column d is read at level >= 1 / = 2
    float knew[kD];                     // fused append: the new token's K row as it will be read at the column levels
    float new_logit[G];                 // fused append: q . knew, accumulated in channel order
};

// Rule 1 for the 128 columns of (b, h), in two steps so that a caller can put other loads in flight between the
// issue of the loads here and their first use.  Both are called by every thread of a workgroup of at least 128
// threads (the second contains barriers); afterwards ks holds q as fp32 and the level masks.
// k_new_bits: fp16 bits of channel tid of a token that is being appended in the same kernel (fused append),
// else -1: K_colmax then counts that token, and the token's row, read at the column levels, is left in
// ks.knew for new_token_logit().
template <int G>
struct KLevelsIn {
    uint32_t cm;         // K_colmax of channel tid as stored
    uint32_t qbits[G];   // fp16 bits of q[g][tid]
};

template <int G>
__device__ __forceinline__ void k_levels_load(const DecodeArgs& a, int b, int h, KLevelsIn<G>& in)
{
    const int tid = threadIdx.x;
    const size_t bh = size_t(b) * a.s.Hkv + h;
    in.cm = 0;
#pragma unroll
    for (int g = 0; g < G; ++g) in.qbits[g] = 0;
    if (tid < kD) {
        in.cm = a.colmax[bh * kD + tid];
#pragma unroll
        for (int g = 0; g < G; ++g) in.qbits[g] = a.q[(size_t(b) * a.s.Hq + size_t(h) * G + g) * kD + tid];
    }
}

// Returns the K_colmax of channel tid (tid < 128) that the levels used.
// stat_len: tokens of the sequence the levels apply to (for the counters of akv_stats; used with export_levels).
template <int G>
__device__ __forceinline__ uint32_t k_levels_finish(const DecodeArgs& a, int b, int h, KShared<G>& ks, bool export_levels,
                                                    int k_new_bits, const KLevelsIn<G>& in, int stat_len)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const size_t bh = size_t(b) * a.s.Hkv + h;
    float P[G];
    uint32_t colmax_used = 0;
    if (tid < kD) {   // waves 0 and 1 (wave-uniform): channel tid
        uint32_t cm = in.cm;
        if (k_new_bits >= 0) cm = max(cm, uint32_t(k_new_bits) & 0x7FFFu);
        colmax_used = cm;
        cm = cm < 0x0400u ? 0x0400u : cm;               // below the smallest normal: its places are 2^-14's
        const float cmf = half_bits_to_float(cm);
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float qf = half_bits_to_float(in.qbits[g]);
            ks.q[g][tid] = qf;
            P[g] = qf * cmf;                             // exact: 11-bit x 11-bit significands
            // the maximum over the wave's 64 columns in the vector ALU (LDS atomics of 64 lanes on one address take a
            // cycle per lane of the LDS unit that all workgroups of the compute unit share)
            const int em = wave_max_int(P[g] != 0.0f ? float_exp_field(P[g]) : -1);
            if (lane == 0) ks.emax[wave][g] = em;
        }
    }
    __syncthreads();
    if (tid < kD) {
        int lv = 0;
#pragma unroll
        for (int g = 0; g < G; ++g) {
            if (P[g] != 0.0f) {
                const int emax = max(ks.emax[0][g], ks.emax[1][g]);
                const int l = level_for_mantissa_bits(10 + a.guard_bits - (emax - float_exp_field(P[g])));
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
        if (a.stats && export_levels && lane == 0) {   // 64 columns of this wave: how many at each level, times the tokens
            const unsigned long long n2 = __builtin_popcountll(b2), n1 = __builtin_popcountll(b1) - n2, n = (unsigned long long)stat_len;
            atomicAdd(reinterpret_cast<unsigned long long*>(&a.stats->k_elems[0]), (64ull - n1 - n2) * n);
            atomicAdd(reinterpret_cast<unsigned long long*>(&a.stats->k_elems[1]), n1 * n);
            atomicAdd(reinterpret_cast<unsigned long long*>(&a.stats->k_elems[2]), n2 * n);
        }
        if (k_new_bits >= 0) {   // "Dynamic Quantization": bits that are not read are filled with 100...
            const uint32_t kb = uint32_t(k_new_bits);
            ks.knew[tid] = half_bits_to_float(lv == 2 ? kb : (lv == 1 ? ((kb & 0xFFF0u) | 0x0008u) : ((kb & 0xFF00u) | 0x0080u)));
        }
    }
    __syncthreads();
    return colmax_used;
}

template <int G>
__device__ __forceinline__ uint32_t k_levels(const DecodeArgs& a, int b, int h, KShared<G>& ks, bool export_levels,
                                             int stat_len, int k_new_bits = -1)
{
    KLevelsIn<G> in;
    k_levels_load<G>(a, b, h, in);
    return k_levels_finish<G>(a, b, h, ks, export_levels, k_new_bits, in, stat_len);
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

// One wave, one 256-token block blk of (b, h): lane -> tokens 4*lane .. 4*lane+3 of the block; the logit of a token
// is accumulated in fp32 over channels in ascending order inside its lane (no reduction).
// Channels are processed 8 at a time.  Per group the wave fetches the 2-KB run of K_hi (8 columns x 256 B,
// contiguous in the channel-major block) with two 16-B loads per lane, and the 1-KB runs of K_mid / K_lo with one
// 16-B load per lane each, lane -> (column lane/8, 16 bytes): a column whose level does not ask for a plane is
// left out by sending its 8 lanes out of range (nothing is fetched, zeros come back).  Four vector-memory
// instructions per group instead of one per column and plane: the address unit of a CU takes about as long
// for a 2-byte-per-lane load as for a 16-byte one, and the count of such instructions, not their bytes, bounded
// this pass.  The loaded registers are in "memory order"; they are written to a 4-KB wave-private LDS
// area and read back in "token order" (lane -> its 4 tokens of every column).
// Logits go to a.logits with cache policy `aux` (kAuxSc1 when another workgroup of the same kernel will read
// them) and are left in acc; the maximum over the tile's valid tokens is returned for every query head of the
// group (same value in all lanes).
constexpr int kKU = 8;            // columns per group
constexpr int kKStage = 4096;     // bytes of LDS staging per wave

// HI bytes of the first three groups of a tile, issued before the levels are known (they are always read):
// pre[] is handed to k_tile (use_pre = true) for the same block.
template <bool NT = true>
__device__ __forceinline__ void k_tile_pre(const DecodeArgs& a, int b, int h, int blk, u32x4_t (&pre)[6])
{
    const int lane = threadIdx.x & 63;
    const size_t bh = size_t(b) * a.s.Hkv + h;
    const __amdgpu_buffer_rsrc_t rh = make_rsrc(a.k_hi + (bh * a.s.Ncap + size_t(blk) * kTB) * kD, uint32_t(kTB) * kD);
#pragma unroll
    for (int i = 0; i < 6; ++i) pre[i] = NT ? buf_load_b128_nt(rh, uint32_t(lane) * 16 + i * 1024) : buf_load_b128(rh, uint32_t(lane) * 16 + i * 1024);
}

// NT: the block's bytes are read with the non-temporal hint (they are read once per step); a caller that is about to
// store into the block's lines (fused append) reads that one block without it, so that the lines stay in L2.
// lds_lg: where a kernel keeps the logits of its (sequence, KV head) in LDS (query head g at lds_lg + g * lds_stride
// floats, token t at index t), or NULL: they go to a.logits.  With LDS logits a.logits is written as well only if it
// is the caller's export buffer (a.dbg.logits).
template <int G, bool NT = true>
__device__ __forceinline__ void k_tile(const DecodeArgs& a, int b, int h, int blk, int len, const KShared<G>& ks,
                                       int aux, float (&tile_max)[G], const u32x4_t (&pre)[6], bool use_pre,
                                       float (&acc)[G][4], uint8_t* stage, float* lds_lg = nullptr, int lds_stride = 0)
{
    constexpr int U = kKU;
    constexpr int kAux = NT ? kAuxNt : 0;
    const int lane = threadIdx.x & 63;
    const int Hkv = a.s.Hkv, Hq = a.s.Hq, Ncap = a.s.Ncap;
    const size_t bh = size_t(b) * Hkv + h;
    blk = __builtin_amdgcn_readfirstlane(blk);   // wave-uniform by contract: scalar addressing

#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[g][i] = 0.0f;

    // the level masks live in scalar registers for the whole loop
    const uint64_t nm0 = uniform64(ks.need_mid[0]), nm1 = uniform64(ks.need_mid[1]);
    const uint64_t nl0 = uniform64(ks.need_lo[0]), nl1 = uniform64(ks.need_lo[1]);
    // bits of the U columns starting at d0 (d0 % U == 0, so a group never straddles the two words)
    auto bits_at = [&](uint64_t w0, uint64_t w1, int d0) -> uint32_t {
        return d0 < kD ? (uint32_t)((d0 < 64 ? w0 : w1) >> (d0 & 63)) & ((1u << U) - 1) : 0u;
    };
    const uint8_t* hi_blk = a.k_hi + (bh * Ncap + size_t(blk) * kTB) * kD;
    const uint8_t* mid_blk = a.k_mid + (bh * Ncap + size_t(blk) * kTB) * (kD / 2);
    const uint8_t* lo_blk = a.k_lo + (bh * Ncap + size_t(blk) * kTB) * (kD / 2);
    const uint32_t voff = uint32_t(lane) * 16;
    const uint32_t col = uint32_t(lane) >> 3;   // the column of the group this lane fetches nibbles of

    struct Group {
        u32x4_t h0, h1;   // bytes 16*lane .. +15 of the first / second KB of the HI run (columns 0..3 / 4..7)
        u32x4_t m, l;     // bytes 16*lane .. +15 of the MID / LO run (column lane/8)
    };
    // groups past the last column are issued through descriptors of size zero: nothing is fetched
    auto issue_hi = [&](Group& gr, int d0) {
        const __amdgpu_buffer_rsrc_t rh = make_rsrc(hi_blk, d0 < kD ? uint32_t(kTB) * kD : 0u);
        gr.h0 = __builtin_amdgcn_raw_buffer_load_b128(rh, voff, d0 * kTB, kAux);
        gr.h1 = __builtin_amdgcn_raw_buffer_load_b128(rh, voff + 1024, d0 * kTB, kAux);
    };
    auto issue_nib = [&](Group& gr, int d0) {
        const uint32_t bm = bits_at(nm0, nm1, d0), bl = bits_at(nl0, nl1, d0);
        const uint32_t size = d0 < kD ? uint32_t(kTB) * (kD / 2) : 0u;
        const __amdgpu_buffer_rsrc_t rm = make_rsrc(mid_blk, size), rl = make_rsrc(lo_blk, size);
        const uint32_t base = voff + uint32_t(d0 < kD ? d0 : 0) * (kTB / 2);
        gr.m = __builtin_amdgcn_raw_buffer_load_b128(rm, ((bm >> col) & 1u) ? base : kSkip, 0, kAux);
        gr.l = __builtin_amdgcn_raw_buffer_load_b128(rl, ((bl >> col) & 1u) ? base : kSkip, 0, kAux);
    };
    auto issue = [&](Group& gr, int d0) {
        issue_hi(gr, d0);
        issue_nib(gr, d0);
    };
    auto compute = [&](const Group& gr, int d0) {
        const uint32_t bm = bits_at(nm0, nm1, d0), bl = bits_at(nl0, nl1, d0);
        // memory order -> token order through the wave's LDS area (LDS serves a wave's accesses in order)
        __builtin_amdgcn_wave_barrier();
        *reinterpret_cast<u32x4_t*>(stage + voff) = gr.h0;
        *reinterpret_cast<u32x4_t*>(stage + 1024 + voff) = gr.h1;
        *reinterpret_cast<u32x4_t*>(stage + 2048 + voff) = gr.m;
        *reinterpret_cast<u32x4_t*>(stage + 3072 + voff) = gr.l;
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t hh = *reinterpret_cast<const uint32_t*>(stage + u * kTB + lane * 4);
            const uint32_t mm = *reinterpret_cast<const uint16_t*>(stage + 2048 + u * (kTB / 2) + lane * 2);
            const uint32_t ll = *reinterpret_cast<const uint16_t*>(stage + 3072 + u * (kTB / 2) + lane * 2);
            uint32_t ev, od;   // low bytes of tokens 0,2 / 1,3
            if ((bl >> u) & 1u) {   // all 16 bits read (uniform branch)
                ev = ((mm << 4) & 0xF0F0F0F0u) | (ll & 0x0F0F0F0Fu);
                od = (mm & 0xF0F0F0F0u) | ((ll >> 4) & 0x0F0F0F0Fu);
            } else {                // 12 bits (MID read, fill 1000) or 8 bits (MID word is zero, fill 1000 0000)
                const uint32_t fill = ((bm >> u) & 1u) ? 0x08080808u : 0x80808080u;
                ev = ((mm << 4) & 0xF0F0F0F0u) | fill;
                od = (mm & 0xF0F0F0F0u) | fill;
            }
            const uint32_t p0 = __builtin_amdgcn_perm(hh, ev, 0x06010400u);   // tokens (0,2)
            const uint32_t p1 = __builtin_amdgcn_perm(hh, od, 0x07010500u);   // tokens (1,3)
            const float k[4] = {lo_half(p0), lo_half(p1), hi_half(p0), hi_half(p1)};
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const float qd = ks.q[g][d0 + u];
                // q*k is exact in fp32, so the fused form rounds exactly like multiply-then-add
#pragma unroll
                for (int i = 0; i < 4; ++i) acc[g][i] = fmaf(qd, k[i], acc[g][i]);
            }
        }
        __builtin_amdgcn_wave_barrier();
    };
    // three groups rotate by name: all three are issued before the first is consumed, and a group is issued again
    // as soon as it has been consumed (8 to 12 KB in flight per wave)
    Group A, B, C;
    if (use_pre) {   // uniform: the HI bytes of the first three groups are already in flight (k_tile_pre)
        A.h0 = pre[0];
        A.h1 = pre[1];
        B.h0 = pre[2];
        B.h1 = pre[3];
        C.h0 = pre[4];
        C.h1 = pre[5];
        issue_nib(A, 0);
        issue_nib(B, U);
        issue_nib(C, 2 * U);
    } else {
        issue(A, 0);
        issue(B, U);
        issue(C, 2 * U);
    }
#pragma unroll 1
    for (int d0 = 0; d0 < kD; d0 += 3 * U) {
        compute(A, d0);
        issue(A, d0 + 3 * U);
        if (d0 + U < kD) compute(B, d0 + U);   // kD is not a multiple of 3 * U: the last round is partial
        issue(B, d0 + 4 * U);
        if (d0 + 2 * U < kD) compute(C, d0 + 2 * U);
        issue(C, d0 + 5 * U);
    }

    // ---- logits out, tile maxima -----------------------------------------------------------------
    const int t0 = blk * kTB + lane * 4;
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const size_t hq = size_t(b) * Hq + size_t(h) * G + g;
        const __amdgpu_buffer_rsrc_t rs_lg = make_rsrc(a.logits + hq * Ncap, uint32_t(Ncap) * 4u);
        u32x4_t w;
        w.x = float_bits(acc[g][0]); w.y = float_bits(acc[g][1]);
        w.z = float_bits(acc[g][2]); w.w = float_bits(acc[g][3]);
        if (lds_lg) *reinterpret_cast<u32x4_t*>(lds_lg + g * lds_stride + t0) = w;
        if (!lds_lg || a.dbg.logits) {
            if (aux) __builtin_amdgcn_raw_buffer_store_b128(w, rs_lg, uint32_t(t0) * 4u, 0, kAuxSc1);
            else __builtin_amdgcn_raw_buffer_store_b128(w, rs_lg, uint32_t(t0) * 4u, 0, 0);
        }
        float m = -INFINITY;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (t0 + i < len) m = fmaxf(m, acc[g][i]);
        tile_max[g] = wave_max(m);
    }
}

}  // namespace akv
