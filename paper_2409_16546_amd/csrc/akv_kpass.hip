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
    __shared__ int lvl_s[kD];
    __shared__ int emax_s[G];

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
    if (tid < kD) {
        int lv = 0;
#pragma unroll
        for (int g = 0; g < G; ++g) {
            if (P[g] != 0.0f) {
                const int l = level_for_mantissa_bits(10 + a.guard_bits - (emax_s[g] - float_exp_field(P[g])));
                lv = l > lv ? l : lv;
            }
        }
        if (a.force_level >= 0) lv = a.force_level;
        lvl_s[tid] = lv;
        if (a.dbg.lvlK && blockIdx.x == 0) a.dbg.lvlK[bh * kD + tid] = (uint8_t)lv;
    }
    __syncthreads();
    if (tile * kKTile >= len) return;                   // this wave's tile is beyond the sequence (uniform per wave)

    // ---- streaming pass ---------------------------------------------------------------------------
    const int blk = tile * 2 + (lane >> 5);
    const bool live = blk < NB;                          // Ncap may end after the tile's first block
    const int blk_ld = live ? blk : NB - 1;              // such lanes re-read the last block and store nothing
    const int j0 = (lane & 31) * kKTpl;
    const uint8_t* phi = a.k_hi + ((bh * NB + blk_ld) * kD) * size_t(kTB) + j0;
    const uint8_t* pmid = a.k_mid + ((bh * NB + blk_ld) * kD) * size_t(kTB / 2) + j0 / 2;
    const uint8_t* plo = a.k_lo + ((bh * NB + blk_ld) * kD) * size_t(kTB / 2) + j0 / 2;

    float acc[G][kKTpl];
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
        for (int i = 0; i < kKTpl; ++i) acc[g][i] = 0.0f;

    constexpr int U = 8;   // channels in flight per step
    uint2 hi[U];
    uint32_t mid[U], lo[U];
    auto issue = [&](int d0) {
#pragma unroll
        for (int u = 0; u < U; ++u) hi[u] = *reinterpret_cast<const uint2*>(phi + size_t(d0 + u) * kTB);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int lv = __builtin_amdgcn_readfirstlane(lvl_s[d0 + u]);
            mid[u] = kFill8;                             // level 0: the 8 unread bits are 1000 0000
            lo[u] = lv == 1 ? kFill8 : 0u;               // level 1: the 4 unread bits are 1000
            if (lv >= 1) mid[u] = *reinterpret_cast<const uint32_t*>(pmid + size_t(d0 + u) * (kTB / 2));
            if (lv >= 2) lo[u] = *reinterpret_cast<const uint32_t*>(plo + size_t(d0 + u) * (kTB / 2));
        }
    };
    for (int d0 = 0; d0 < kD; d0 += U) {
        issue(d0);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            uint32_t p[4];
            assemble8(hi[u].x, hi[u].y, mid[u], lo[u], p);
            const float k0 = lo_half(p[0]), k2 = hi_half(p[0]), k1 = lo_half(p[1]), k3 = hi_half(p[1]);
            const float k4 = lo_half(p[2]), k6 = hi_half(p[2]), k5 = lo_half(p[3]), k7 = hi_half(p[3]);
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
