// K side of decode attention: Rule 1 level per K column, then the streaming q.K~ pass.
// "Quantization of K-Cache": from q and K_colmax estimate the magnitude of the 128 addends of one logit,
// align them to the coarsest one (Rule 1), read each column of K at the bit width its addend needs.
#include "akv_common.h"

namespace akv {

// Workgroup = kKWaves waves, one (sequence, KV head); each wave owns one 512-token tile (two K blocks):
// lane -> block (lane / 32) and 8 consecutive tokens; for every channel d the wave reads one contiguous
// 256-B run of K_hi per block and, if the column's level asks for it, the 128-B runs of K_mid / K_lo.
// Every byte is used by exactly one lane, so nothing is staged through LDS; LDS holds q and the levels.
// The logit of a token is accumulated in fp32 over channels in ascending order (one lane, no reduction).
template <int G>
__global__ __launch_bounds__(64 * kKWaves) void kpass_kernel(DecodeArgs a)
{
    __shared__ float q_s[G][kD];
    __shared__ int emax_s[G];
    __shared__ uint64_t need_mid_s[2], need_lo_s[2];   // bit d%64 of word d/64: column d is read at level >= 1 / = 2

    const int h = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int Hkv = a.s.Hkv, Hq = a.s.Hq, Ncap = a.s.Ncap, NB = Ncap / kTB;
    const int len = min(a.lens[b], Ncap);
    const size_t bh = size_t(b) * Hkv + h;
    const int tile = blockIdx.x * kKWaves + wave;       // 512-token tile of this wave
    if (blockIdx.x * kKTokensPerWg >= len) return;      // whole workgroup beyond the sequence (uniform)

    // ---- Rule 1: level per column -------------------------------------------------------------
    if (tid < G) emax_s[tid] = -1;
    __syncthreads();
    float P[G];
    if (tid < kD) {
        uint32_t cm = a.colmax[bh * kD + tid];
        cm = cm < 0x0400u ? 0x0400u : cm;               // below the smallest normal: its places are 2^-14's
        const float cmf = half_bits_to_float(cm);
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float qf = half_bits_to_float(a.q[(size_t(b) * Hq + size_t(h) * G + g) * kD + tid]);
            q_s[g][tid] = qf;
            P[g] = qf * cmf;                             // exact: 11-bit x 11-bit significands
            if (P[g] != 0.0f) atomicMax(&emax_s[g], float_exp_field(P[g]));
        }
    }
    __syncthreads();
    if (tid < kD) {   // waves 0 and 1: channel tid
        int lv = 0;
#pragma unroll
        for (int g = 0; g < G; ++g) {
            if (P[g] != 0.0f) {
                const int l = level_for_mantissa_bits(10 + a.guard_bits - (emax_s[g] - float_exp_field(P[g])));
                lv = l > lv ? l : lv;
            }
        }
        if (a.force_level >= 0) lv = a.force_level;
        const uint64_t b1 = __ballot(lv >= 1), b2 = __ballot(lv >= 2);
        if (lane == 0) {
            need_mid_s[wave] = b1;
            need_lo_s[wave] = b2;
        }
        if (a.dbg.lvlK && blockIdx.x == 0) a.dbg.lvlK[bh * kD + tid] = (uint8_t)lv;
    }
    __syncthreads();
    if (tile * kKTile >= len) return;                   // this wave's tile is beyond the sequence (uniform per wave)

    // ---- streaming pass ---------------------------------------------------------------------------
    // Channels go in groups of U; the loads of group i+1 are issued before the arithmetic of group i.  A
    // column whose level does not ask for MID / LO gets the offset kSkip: the load returns zero and fetches
    // nothing, and the fill for the unread bits is OR-ed in.
    const int blk = tile * 2 + (lane >> 5);
    const bool live = blk < NB;                          // Ncap may end after the tile's first block
    const int blk_ld = live ? blk : NB - 1;              // such lanes re-read the last block and store nothing
    const int j0 = (lane & 31) * kKTpl;
    const uint32_t off_hi = uint32_t(blk_ld) * kD * kTB + j0;
    const uint32_t off_nib = uint32_t(blk_ld) * kD * (kTB / 2) + j0 / 2;

    float acc[G][kKTpl];
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
        for (int i = 0; i < kKTpl; ++i) acc[g][i] = 0.0f;

    // the level masks live in scalar registers for the whole loop
    auto uniform64 = [](uint64_t v) -> uint64_t {   // readfirstlane returns a signed int: widen through uint32_t
        const uint32_t lo32 = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
        const uint32_t hi32 = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(v >> 32));
        return (uint64_t(hi32) << 32) | uint64_t(lo32);
    };
    const uint64_t nm0 = uniform64(need_mid_s[0]), nm1 = uniform64(need_mid_s[1]);
    const uint64_t nl0 = uniform64(need_lo_s[0]), nl1 = uniform64(need_lo_s[1]);

    constexpr int U = 8;   // channels per group
    struct Group {
        u32x2_t h[U];
        uint32_t m[U], l[U];
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
            gr.h[u] = __builtin_amdgcn_raw_buffer_load_b64(rh, off_hi + u * kTB, d0 * kTB, 0);
            gr.m[u] = __builtin_amdgcn_raw_buffer_load_b32(rm, off_nib + u * (kTB / 2), d0 * (kTB / 2), 0);
            gr.l[u] = __builtin_amdgcn_raw_buffer_load_b32(rl, off_nib + u * (kTB / 2), d0 * (kTB / 2), 0);
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
            const uint32_t p0 = __builtin_amdgcn_perm(gr.h[u].x, ev, 0x06010400u);   // tokens (0,2)
            const uint32_t p1 = __builtin_amdgcn_perm(gr.h[u].x, od, 0x07010500u);   // tokens (1,3)
            const uint32_t p2 = __builtin_amdgcn_perm(gr.h[u].y, ev, 0x06030402u);   // tokens (4,6)
            const uint32_t p3 = __builtin_amdgcn_perm(gr.h[u].y, od, 0x07030502u);   // tokens (5,7)
            const float k0 = lo_half(p0), k2 = hi_half(p0), k1 = lo_half(p1), k3 = hi_half(p1);
            const float k4 = lo_half(p2), k6 = hi_half(p2), k5 = lo_half(p3), k7 = hi_half(p3);
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const float qd = q_s[g][d0 + u];
                // q*k is exact in fp32, so the fused form rounds exactly like multiply-then-add
                acc[g][0] = fmaf(qd, k0, acc[g][0]);
                acc[g][1] = fmaf(qd, k1, acc[g][1]);
                acc[g][2] = fmaf(qd, k2, acc[g][2]);
                acc[g][3] = fmaf(qd, k3, acc[g][3]);
                acc[g][4] = fmaf(qd, k4, acc[g][4]);
                acc[g][5] = fmaf(qd, k5, acc[g][5]);
                acc[g][6] = fmaf(qd, k6, acc[g][6]);
                acc[g][7] = fmaf(qd, k7, acc[g][7]);
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
        if (d0 + U < kD) compute(B, d0 + U);
        issue(B, d0 + 4 * U);
        if (d0 + 2 * U < kD) compute(C, d0 + 2 * U);
    }

    // ---- logits out, tile maxima -----------------------------------------------------------------
    const int t0 = blk * kTB + j0;
    const int ntile = k_tiles(Ncap);
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const size_t hq = size_t(b) * Hq + size_t(h) * G + g;
        float* dst = a.logits + hq * Ncap + t0;
        if (live) {
            *reinterpret_cast<float4*>(dst) = make_float4(acc[g][0], acc[g][1], acc[g][2], acc[g][3]);
            *reinterpret_cast<float4*>(dst + 4) = make_float4(acc[g][4], acc[g][5], acc[g][6], acc[g][7]);
        }
        float m = -INFINITY;
#pragma unroll
        for (int i = 0; i < kKTpl; ++i)
            if (live && t0 + i < len) m = fmaxf(m, acc[g][i]);
        m = wave_max(m);
        if (lane == 0) a.tilemax[hq * ntile + tile] = m;
    }
}

hipError_t launch_kpass(const DecodeArgs& a, hipStream_t st)
{
    const int G = a.s.Hq / a.s.Hkv;
    const dim3 grid((a.max_len + kKTokensPerWg - 1) / kKTokensPerWg, a.s.Hkv, a.s.B), block(64 * kKWaves);
    switch (G) {
        case 1: hipLaunchKernelGGL(kpass_kernel<1>, grid, block, 0, st, a); break;
        case 2: hipLaunchKernelGGL(kpass_kernel<2>, grid, block, 0, st, a); break;
        case 4: hipLaunchKernelGGL(kpass_kernel<4>, grid, block, 0, st, a); break;
        case 8: hipLaunchKernelGGL(kpass_kernel<8>, grid, block, 0, st, a); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace akv
