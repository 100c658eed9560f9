// Decode attention, token-split path: the tokens of every (sequence, KV head) are spread over many
// workgroups (long contexts, few heads).  Two kernels:
//   K kernel  Rule 1 levels + q.K~, one 256-token block per wave; the workgroup of a (sequence, KV head) that
//             finishes last runs the mid step (max, score exponents, top-k, O_est, result exponents);
//   V kernel  Rule 2 + S.V~ over 512-token chunks; the workgroup that finishes last combines the chunks.
// Sections "Quantization of K-Cache", "Quantization of V-Cache", "Runtime of AlignedKV".
#include "akv_common.h"
#include "akv_k_tile.h"
#include "akv_mid_step.h"
#include "akv_v_rows.h"

namespace akv {

template <int G>
__global__ __launch_bounds__(64 * kKWaves) void split_k_kernel(DecodeArgs a)
{
    constexpr int kTile = kTB;   // tokens per wave
    __shared__ __align__(16) uint8_t kstage[kKWaves][kKStage];
    __shared__ KShared<G> ks;
    __shared__ MidShared ms;
    __shared__ float red_s[G][kKWaves];
    __shared__ int last_s;

    const int h = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int Hkv = a.s.Hkv, Hq = a.s.Hq, Ncap = a.s.Ncap, NB = Ncap / kTB;
    const int len = min(a.lens[b], Ncap);
    const size_t bh = size_t(b) * Hkv + h;
    const int tile = blockIdx.x * kKWaves + __builtin_amdgcn_readfirstlane(wave);
    if (blockIdx.x * (kTile * kKWaves) >= len) return;   // whole workgroup beyond the sequence (uniform)

    k_levels<G>(a, b, h, ks, blockIdx.x == 0);
    if (tile * kTile < len) {                            // else this wave's tile is beyond the sequence
        float tm[G];
        const u32x4_t zero4 = {0u, 0u, 0u, 0u};
        const u32x4_t none[4] = {zero4, zero4, zero4, zero4};
        float lg[G][4];
        k_tile<G>(a, b, h, tile, len, ks, kAuxSc1, tm, none, false, lg, &kstage[__builtin_amdgcn_readfirstlane(wave)][0]);
        if (lane == 0)
#pragma unroll
            for (int g = 0; g < G; ++g)   // NB slots per head: one per block
                store_agent(&a.tilemax[(size_t(b) * Hq + size_t(h) * G + g) * NB + tile], tm[g]);
    }

    // ---- the workgroup that finishes last for this (sequence, KV head) runs the mid step ------------
    // Every workgroup waits until its device-scope stores are acknowledged and takes a ticket; the one that
    // draws the last ticket reads all logits at device scope.  Nobody waits for anybody.
    stores_done();
    __syncthreads();
    if (tid == 0) {
        const int nwg = (len + kTile * kKWaves - 1) / (kTile * kKWaves);
        last_s = take_ticket(&a.kcount[bh]) == nwg - 1;
    }
    __syncthreads();
    if (!last_s) return;
    // M = max over the tile maxima (exact, order-free)
    const int ntiles = (len + kTile - 1) / kTile;
#pragma unroll
    for (int g = 0; g < G; ++g) {
        float m = -INFINITY;
        for (int i = tid; i < ntiles; i += 64 * kKWaves)
            m = fmaxf(m, load_agent(&a.tilemax[(size_t(b) * Hq + size_t(h) * G + g) * NB + i]));
        m = wave_max(m);
        if (lane == 0) red_s[g][wave] = m;
    }
    __syncthreads();
    if (tid < G) {
        float m = red_s[tid][0];
        for (int w = 1; w < kKWaves; ++w) m = fmaxf(m, red_s[tid][w]);
        ms.M[tid] = m;
    }
    __syncthreads();
    const float none4[G][4] = {};
    mid_step<G, 64 * kKWaves, true>(a, b, h, len, ms, none4, false);
    if (tid == 0) store_agent(&a.kcount[bh], 0);   // ready for the next call
}

// Workgroup = kVWaves waves, one (sequence, KV head, 512-token chunk); wave w takes the batches of 32 rows
// w, w + kVWaves, ... of the chunk.
template <int G, bool DEBUG>
__global__ __launch_bounds__(64 * kVWaves) void split_v_kernel(DecodeArgs a)
{
    __shared__ float red_s[kVWaves][G][kD + 1];
    __shared__ int last_s;

    const int h = blockIdx.y, b = blockIdx.z, split = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = lane >> 3, cl = lane & 7;
    const int Hkv = a.s.Hkv, Hq = a.s.Hq, Ncap = a.s.Ncap;
    const int len = min(a.lens[b], Ncap);
    const int c0 = split * kVChunk;
    const size_t bh = size_t(b) * Hkv + h;
    const int nsplit = v_splits(Ncap);
    if (c0 >= len) {                                    // uniform: chunk beyond the sequence
        if (len == 0 && split == 0)                     // an empty sequence attends to nothing: zeros
            for (int idx = tid; idx < G * kD; idx += 64 * kVWaves)
                store_out(a, size_t(b) * Hq + size_t(h) * G + idx / kD, idx % kD, 0.0f);
        return;
    }

    VRule vr;
    v_rule_setup(a.Ehat + bh * kD, a.guard_bits, a.force_level, vr);
    float Mg[G];
#pragma unroll
    for (int g = 0; g < G; ++g) Mg[g] = a.M[size_t(b) * Hq + size_t(h) * G + g];
    float acc[G][16], z[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        z[g] = 0.0f;
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[g][i] = 0.0f;
    }
    const u32x4_t none[1][4] = {};
    v_rows<G, 4, DEBUG, 0>(a, b, h, c0 + wave * 32, 32 * kVWaves, kVChunk / (32 * kVWaves), len, vr, Mg, acc, z, none, false);
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
    for (int idx = tid; idx < G * (kD + 1); idx += 64 * kVWaves) {
        const int g = idx / (kD + 1), d = idx % (kD + 1);
        float s = 0.0f;
#pragma unroll
        for (int w = 0; w < kVWaves; ++w) s += red_s[w][g][d];
        const size_t hq = size_t(b) * Hq + size_t(h) * G + g;
        if (d < kD) store_agent(&a.partO[(hq * nsplit + split) * kD + d], s);
        else store_agent(&a.partZ[hq * nsplit + split], s);
    }

    // ---- the workgroup that finishes last for this (sequence, KV head) combines the chunks -------------
    // out = sum_chunks O / sum_chunks Z: every chunk used the same global max, so nothing is rescaled.
    const int used = v_splits(len);
    stores_done();
    __syncthreads();
    if (tid == 0) last_s = take_ticket(&a.vcount[bh]) == used - 1;
    __syncthreads();
    if (!last_s) return;
    for (int idx = tid; idx < G * kD; idx += 64 * kVWaves) {
        const int g = idx / kD, d = idx % kD;
        const size_t hq = size_t(b) * Hq + size_t(h) * G + g;
        float o = 0.0f, zsum = 0.0f;
        for (int sp = 0; sp < used; ++sp) {
            o += load_agent(&a.partO[(hq * nsplit + sp) * kD + d]);
            zsum += load_agent(&a.partZ[hq * nsplit + sp]);
        }
        store_out(a, hq, d, o / zsum);
    }
    if (tid == 0) store_agent(&a.vcount[bh], 0);   // ready for the next call
}

template <int G>
static hipError_t launch_split_g(const DecodeArgs& a, hipStream_t st, hipEvent_t mid_event)
{
    const int tile = kTB * kKWaves;   // tokens per workgroup of the K kernel: one 256-token block per wave
    const dim3 kgrid((a.max_len + tile - 1) / tile, a.s.Hkv, a.s.B), kblock(64 * kKWaves);
    hipLaunchKernelGGL((split_k_kernel<G>), kgrid, kblock, 0, st, a);
    if (hipError_t e = hipGetLastError()) return e;
    if (mid_event)
        if (hipError_t e = hipEventRecord(mid_event, st)) return e;
    const dim3 vgrid(v_splits(a.max_len), a.s.Hkv, a.s.B), vblock(64 * kVWaves);
    if (a.dbg.needV || a.dbg.appliedV) hipLaunchKernelGGL((split_v_kernel<G, true>), vgrid, vblock, 0, st, a);
    else hipLaunchKernelGGL((split_v_kernel<G, false>), vgrid, vblock, 0, st, a);
    return hipGetLastError();
}

hipError_t launch_decode_split(const DecodeArgs& a, hipStream_t st, hipEvent_t mid_event)
{
    switch (a.s.Hq / a.s.Hkv) {
        case 1: return launch_split_g<1>(a, st, mid_event);
        case 2: return launch_split_g<2>(a, st, mid_event);
        case 4: return launch_split_g<4>(a, st, mid_event);
        case 8: return launch_split_g<8>(a, st, mid_event);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace akv
