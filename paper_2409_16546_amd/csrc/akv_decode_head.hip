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

// lens[b] is shared by the heads of a sequence.  Every workgroup reads it at its start and then takes a ticket
// (the atomic's result is not looked at before the end of the kernel, so nothing waits for it); the one that
// drew the last ticket -- every head has read the old length by then -- stores the new length at its end, or
// counts the refusal.
__device__ __forceinline__ void finish_append(const DecodeArgs& a, int b, int len_old, int ticket)
{
    if (!a.k_new || threadIdx.x != 0) return;
    if (ticket == a.s.Hkv - 1) {
        store_agent(&a.flags[AKV_NFLAGS + b], 0);
        if (len_old + 1 <= a.s.Ncap) const_cast<int32_t*>(a.lens)[b] = len_old + 1;
        else atomicAdd(&a.flags[AKV_FLAG_OVERFLOW], 1);
    }
}

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
    const int Hq = a.s.Hq, Hkv = a.s.Hkv, Ncap = a.s.Ncap;
    const size_t bh = size_t(b) * Hkv + h;
    __shared__ int len_s;
    int ticket = -1;
    if (tid == 0) {
        len_s = min(a.lens[b], Ncap);
        if (a.k_new) {
            stores_done();   // the length has been read (and parked in LDS) before the ticket is taken
            ticket = take_ticket(&a.flags[AKV_NFLAGS + b]);
        }
    }
    __syncthreads();
    const int len_old = len_s;
    const bool appended = a.k_new && len_old + 1 <= Ncap;   // a full sequence keeps its tokens (counted at the end)
    // Fused append of one token: this workgroup owns every byte of (b, h).  The K side below runs over the
    // len_old tokens already stored and takes the new token's logit from its fp16 row directly, so nothing
    // waits for the plane stores; they are issued after the K tiles and are long complete when the V side
    // reads row len_old.
    int k_new_bits = -1;
    uint32_t old_m = 0, old_l = 0;   // the nibble bytes the new token shares with its neighbour
    if (appended && tid < kD) {
        k_new_bits = a.k_new[bh * kD + tid];
        const size_t nib = k_nibble_index(bh, Ncap, len_old, tid);
        old_m = a.k_mid[nib];   // in flight together with the loads of the level computation
        old_l = a.k_lo[nib];
    }
    const int len = len_old + (appended ? 1 : 0);
    if (len == 0) {                                     // an empty sequence attends to nothing: zeros
        for (int idx = tid; idx < G * kD; idx += NT) store_out(a, size_t(b) * Hq + size_t(h) * G + idx / kD, idx % kD, 0.0f);
        finish_append(a, b, len_old, ticket);
        return;
    }

    // ---- K side: levels, then the tiles of the head round-robin over the waves ----------------------
    const uint32_t colmax_used = k_levels<G>(a, b, h, ks, true, k_new_bits);
    if (appended && tid >= NT - 64 && tid < NT - 64 + G) {   // a lane of the last wave per query head
        const int g = tid - (NT - 64);
        ks.new_logit[g] = new_token_logit<G>(ks, g);
    }
    float wm[G];
#pragma unroll
    for (int g = 0; g < G; ++g) wm[g] = -INFINITY;
    // The 256-token blocks of the head are dealt out in contiguous, balanced ranges (sizes differ by at most
    // one block); a wave walks its range two blocks at a time (512-token tiles), then a last single block,
    // so that e.g. 17 blocks on 16 waves still take one tile's time.
    const int nblk = (len_old + kTB - 1) / kTB;   // the tokens already stored
    const int per = nblk / kWaves, extra = nblk % kWaves;
    int blk = wave * per + min(wave, extra);
    const int blk_end = blk + per + (wave < extra ? 1 : 0);
    while (blk < blk_end) {
        float tm[G];
        if (blk + 2 <= blk_end) {
            k_tile<G, 8, 4>(a, b, h, blk, len_old, ks, 0, tm);
            blk += 2;
        } else {
            k_tile<G, 4, 8>(a, b, h, blk, len_old, ks, 0, tm);
            blk += 1;
        }
#pragma unroll
        for (int g = 0; g < G; ++g) wm[g] = fmaxf(wm[g], tm[g]);
    }
    if (lane == 0)
#pragma unroll
        for (int g = 0; g < G; ++g) wmax_s[g][wave] = wm[g];
    if (appended && tid < kD) {   // the new token goes into the planes (the block's lines were just read: they are in L2), K_colmax follows
        store_token_rmw(const_cast<uint8_t*>(a.k_hi), const_cast<uint8_t*>(a.k_mid), const_cast<uint8_t*>(a.k_lo),
                        const_cast<uint8_t*>(a.v_hi), const_cast<uint8_t*>(a.v_mid), const_cast<uint8_t*>(a.v_lo), bh,
                        Ncap, len_old, tid, a.k_new + bh * kD, a.v_new + bh * kD, old_m, old_l);
        const_cast<uint16_t*>(a.colmax)[bh * kD + tid] = (uint16_t)colmax_used;
    }
    __syncthreads();   // also: every logit store and the new token's bytes have completed (same CU, same L2)
    if (tid < G) {
        float m = -INFINITY;
        if (appended) {   // after the barrier: the tile that covers position len_old has stored its vector
            m = ks.new_logit[tid];
            a.logits[(size_t(b) * Hq + size_t(h) * G + tid) * Ncap + len_old] = m;
        }
        for (int w = 0; w < kWaves; ++w) m = fmaxf(m, wmax_s[tid][w]);
        ms.M[tid] = m;
    }
    __syncthreads();

    // ---- mid step -----------------------------------------------------------------------------------
    mid_step<G, NT, false>(a, b, h, len, ms);

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
    finish_append(a, b, len_old, ticket);
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
