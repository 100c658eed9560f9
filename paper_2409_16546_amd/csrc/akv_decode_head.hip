// Decode attention, head-per-workgroup path: ONE workgroup does everything for one (sequence, KV head) --
// Rule 1 levels, q.K~ over all tiles, the mid step, Rule 2 + S.V~ over all rows, the final division --
// so nothing is handed between workgroups and one launch covers the whole step.  Used when there are enough
// (sequence, KV head) pairs to fill the chip.  Logits live in the workspace (they stay in this XCD's L2).
// Sections "Quantization of K-Cache", "Quantization of V-Cache", "Runtime of AlignedKV".
#include "akv_common.h"
#include "akv_k_tile.h"
#include "akv_mid_step.h"
#include "akv_v_rows.h"

namespace akv {

template <int G, int NT, bool DEBUG>
__global__ __launch_bounds__(NT) void head_kernel(DecodeArgs a)
{
    constexpr int kWaves = NT / 64;
    __shared__ KShared<G> ks;
    __shared__ MidShared ms;
    __shared__ float wmax_s[G][kWaves];
    __shared__ float red_s[kWaves][G][kD + 1];

    const int h = blockIdx.x, b = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = lane >> 3, cl = lane & 7;
    const int Hq = a.s.Hq, Ncap = a.s.Ncap;
    const int len = min(a.lens[b], Ncap);
    if (len == 0) {                                     // an empty sequence attends to nothing: zeros
        for (int idx = tid; idx < G * kD; idx += NT) store_out(a, size_t(b) * Hq + size_t(h) * G + idx / kD, idx % kD, 0.0f);
        return;
    }

    // ---- K side: levels, then the tiles of the head round-robin over the waves ----------------------
    k_levels<G>(a, b, h, ks, true);
    float wm[G];
#pragma unroll
    for (int g = 0; g < G; ++g) wm[g] = -INFINITY;
    // The 256-token blocks of the head are dealt out in contiguous, balanced ranges (sizes differ by at most
    // one block); a wave walks its range two blocks at a time (512-token tiles), then a last single block,
    // so that e.g. 17 blocks on 16 waves still take one tile's time.
    const int nblk = (len + kTB - 1) / kTB;
    const int per = nblk / kWaves, extra = nblk % kWaves;
    int blk = wave * per + min(wave, extra);
    const int blk_end = blk + per + (wave < extra ? 1 : 0);
    while (blk < blk_end) {
        float tm[G];
        if (blk + 2 <= blk_end) {
            k_tile<G, 8, 4>(a, b, h, blk, len, ks, 0, tm);
            blk += 2;
        } else {
            k_tile<G, 4, 8>(a, b, h, blk, len, ks, 0, tm);
            blk += 1;
        }
#pragma unroll
        for (int g = 0; g < G; ++g) wm[g] = fmaxf(wm[g], tm[g]);
    }
    if (lane == 0)
#pragma unroll
        for (int g = 0; g < G; ++g) wmax_s[g][wave] = wm[g];
    __syncthreads();   // also: every logit store of the workgroup has completed (same CU, same L2)
    if (tid < G) {
        float m = wmax_s[tid][0];
        for (int w = 1; w < kWaves; ++w) m = fmaxf(m, wmax_s[tid][w]);
        ms.M[tid] = m;
    }
    __syncthreads();

    // ---- mid step -----------------------------------------------------------------------------------
    mid_step<G, NT, false>(a, b, h, ms);

    // ---- V side: batches of 32 rows round-robin over the waves ----------------------------------------
    VRule vr;
    v_rule_setup(ms.ehat, a.guard_bits, vr);
    float Mg[G];
#pragma unroll
    for (int g = 0; g < G; ++g) Mg[g] = ms.M[g];
    float acc[G][16], z[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        z[g] = 0.0f;
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[g][i] = 0.0f;
    }
    const int nbatch = (len + 31) / 32;
    const int mine = nbatch > wave ? (nbatch - wave + kWaves - 1) / kWaves : 0;
    v_rows<G, DEBUG>(a, b, h, wave * 32, 32 * kWaves, mine, len, vr, Mg, acc, z);
    v_reduce_rows<G>(acc, z);
    if (r == 0) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
#pragma unroll
            for (int i = 0; i < 16; ++i) red_s[wave][g][cl * 16 + i] = acc[g][i];
            if (cl == 0) red_s[wave][g][kD] = z[g];
        }
    }
    __syncthreads();
    for (int idx = tid; idx < G * kD; idx += NT) {
        const int g = idx / kD, d = idx % kD;
        float o = 0.0f, zsum = 0.0f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            o += red_s[w][g][d];
            zsum += red_s[w][g][kD];
        }
        store_out(a, size_t(b) * Hq + size_t(h) * G + g, d, o / zsum);
    }
}

template <int G, int NT>
static hipError_t launch_head_g(const DecodeArgs& a, hipStream_t st)
{
    const dim3 grid(a.s.Hkv, a.s.B), block(NT);
    if (a.dbg.needV || a.dbg.appliedV) hipLaunchKernelGGL((head_kernel<G, NT, true>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((head_kernel<G, NT, false>), grid, block, 0, st, a);
    return hipGetLastError();
}

bool head_path_supported(const akv_shape& s) { return s.Hq / s.Hkv <= 4; }

hipError_t launch_decode_head(const DecodeArgs& a, hipStream_t st)
{
    switch (a.s.Hq / a.s.Hkv) {
        case 1: return launch_head_g<1, 1024>(a, st);
        case 2: return launch_head_g<2, 512>(a, st);
        case 4: return launch_head_g<4, 512>(a, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace akv
