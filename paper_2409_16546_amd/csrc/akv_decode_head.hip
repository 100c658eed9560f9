// Decode attention, head-per-workgroup path: ONE workgroup does everything for one (sequence, KV head) --
// Rule 1 levels, q.K~ over all tiles, the mid step, Rule 2 + S.V~ over all rows, the final division --
// so nothing is handed between workgroups and one launch covers the whole step.  Used when there are enough
// (sequence, KV head) pairs to fill the chip.  Logits live in the workspace (they stay in this XCD's L2).
// Workgroup L of the launch runs on XCD L % 8; an XCD takes consecutive pairs (4.5 % faster than every eighth pair).
// Sections "Quantization of K-Cache", "Quantization of V-Cache", "Runtime of AlignedKV".
#include "akv_common.h"
#include "akv_k_tile.h"
#include "akv_mid_step.h"
#include "akv_v_rows.h"

#include <algorithm>

namespace akv {

// lens[b] is shared by the heads of a sequence.  Every workgroup reads it at its start and takes a ticket
// later (thread 0, once its wave is done with its K tile and would otherwise idle at the barrier: the
// round trip of the atomic costs nothing there); the one that drew the last ticket -- every head has read the
// old length by then -- stores the new length at its end, or counts the refusal.
__device__ __forceinline__ void finish_append(const DecodeArgs& a, int b, int len_old, int ticket)
{
    if (!a.k_new || threadIdx.x != 0) return;
    if (ticket == a.s.Hkv - 1) {
        store_agent(&a.flags[AKV_NFLAGS + b], 0);
        if (len_old + 1 <= a.s.Ncap) const_cast<int32_t*>(a.lens)[b] = len_old + 1;
        else atomicAdd(&a.flags[AKV_FLAG_OVERFLOW], 1);
    }
}

// batches of V rows whose HI bytes a wave fetches while it waits for the mid step, and keeps in flight afterwards
// (three where the registers allow it: 1.7 % faster than two on 4096 tokens; four spill)
template <int G> constexpr int head_v_pre() { return G == 1 ? 3 : 2; }
// groups of 8 rows per batch of the V side: what the register budget of the launch shape allows
template <int G, int NT> constexpr int head_v_groups() { return NT <= 512 && G <= 2 ? 4 : 2; }

// LDSLG: the logits of the pair stay in LDS (lds_tokens floats per query head, dynamic shared memory) between the K
// side, the mid step and the V side instead of going through the workspace: nothing of them is written to memory
// (16 MB of logits written during a 0.8 GB stream cost as much time as 100 MB of reads on this machine).
extern __shared__ __align__(16) float head_lds_logits[];

template <int G, int NT, bool DEBUG, bool LDSLG>
__global__ __launch_bounds__(NT) void head_kernel(DecodeArgs a, int lds_tokens)
{
    constexpr int kWaves = NT / 64;
    float* const lds_lg = LDSLG ? head_lds_logits : nullptr;
    __shared__ KShared<G> ks;
    __shared__ MidShared ms;
    __shared__ float wmax_s[G][kWaves];
    __shared__ float red_s[kWaves][G][kD + 1];
    __shared__ __align__(16) uint8_t kstage[kWaves][kKStage];

    const int Hq = a.s.Hq, Hkv = a.s.Hkv, Ncap = a.s.Ncap;
    const int pair = xcd_work_index(blockIdx.x, gridDim.x);   // an XCD takes consecutive heads
    if (pair >= a.s.B * Hkv) return;
    const int h = pair % Hkv, b = pair / Hkv;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = lane >> 3, cl = lane & 7;
    const size_t bh = size_t(b) * Hkv + h;
    int ticket = -1;
    // q and K_colmax of the head are asked for first: everything below queues up behind them
    KLevelsIn<G> lin;
    k_levels_load<G>(a, b, h, lin);
    int k_new_raw = 0;   // fused append: channel tid of the new token's K row (its use waits for the length)
    if (a.k_new && tid < kD) k_new_raw = a.k_new[bh * kD + tid];
    // the same address in every lane: a scalar load, the length lives in a scalar register
    const int len_old = __builtin_amdgcn_readfirstlane(min(a.lens[b], Ncap));
    const bool appended = a.k_new && len_old + 1 <= Ncap;   // a full sequence keeps its tokens (counted at the end)
    // Fused append of one token: this workgroup owns every byte of (b, h).  The K side below runs over the
    // len_old tokens already stored and takes the new token's logit from its fp16 row directly, so nothing
    // waits for the plane stores; they are issued after the K tiles and are long complete when the V side
    // reads row len_old.
    int k_new_bits = -1;
    uint32_t old_m = 0, old_l = 0;   // the nibble bytes the new token shares with its neighbour
    if (appended && tid < kD) {
        k_new_bits = k_new_raw;
        if (len_old & 1) {   // an even place opens its nibble byte (never written: zero), an odd one shares it with the token before
            const size_t nib = k_nibble_index(bh, Ncap, len_old, tid);
            old_m = a.k_mid[nib];   // in flight together with the loads of the level computation
            old_l = a.k_lo[nib];
        }
    }
    // A sequence longer than the caller's bound max_len is attended over its first max_len tokens (as on the
    // token-split path) and counted; the new token is stored in any case.
    const int len_k = min(len_old, a.max_len);                      // stored tokens the K side walks
    const bool attend_new = appended && len_old + 1 <= a.max_len;   // the new token takes part in the attention
    const int len = len_k + (attend_new ? 1 : 0);
    if (h == 0 && tid == 0 && len_old + (appended ? 1 : 0) > a.max_len) atomicAdd(&a.flags[AKV_FLAG_MAXLEN], 1);
    if (len == 0) {                                     // an empty sequence attends to nothing: zeros
        for (int idx = tid; idx < G * kD; idx += NT) store_out(a, size_t(b) * Hq + size_t(h) * G + idx / kD, idx % kD, 0.0f);
        finish_append(a, b, len_old, ticket);
        return;
    }

    // ---- K side: levels, then the 256-token blocks of the head dealt over the waves ---------------------
    // in contiguous, balanced ranges (sizes differ by at most one block)
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const int nblk = (len_k + kTB - 1) / kTB;   // the tokens already stored
    const int per = nblk / kWaves, extra = nblk % kWaves;
    int blk = wave_u * per + min(wave_u, extra);
    const int blk_end = blk + per + (wave_u < extra ? 1 : 0);
    // The HI bytes of the wave's first block do not depend on the levels: they go in flight behind the loads of
    // the level computation (issued at the top of the kernel) and arrive while it runs.
    const u32x4_t zero4 = {0u, 0u, 0u, 0u};
    u32x4_t kpre[6] = {zero4, zero4, zero4, zero4, zero4, zero4};
    const bool pre_any = blk < blk_end;
    // the block the new token goes into is read without the non-temporal hint: its lines stay in L2 for the stores
    const int keep_blk = appended ? len_old / kTB : -1;
    if (pre_any) {
        if (blk == keep_blk) k_tile_pre<false>(a, b, h, blk, kpre);
        else k_tile_pre<true>(a, b, h, blk, kpre);
    }
    const uint32_t colmax_used = k_levels_finish<G>(a, b, h, ks, true, k_new_bits, lin, len);
    float wm[G];
#pragma unroll
    for (int g = 0; g < G; ++g) wm[g] = -INFINITY;
    auto fold = [&](const float (&tm)[G]) {
#pragma unroll
        for (int g = 0; g < G; ++g) wm[g] = fmaxf(wm[g], tm[g]);
    };
    // own[g][i]: logit of token 4*tid + i if the wave's only block was block `wave` (at most kWaves blocks: the
    // mid step then takes its logits from these registers instead of reading them back)
    float own[G][4];
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
        for (int i = 0; i < 4; ++i) own[g][i] = 0.0f;
    uint8_t* stage = &kstage[wave_u][0];
    if (pre_any) {   // the block whose first HI bytes are already in flight
        float tm[G];
        if (blk == keep_blk) k_tile<G, false>(a, b, h, blk, len_k, ks, 0, tm, kpre, true, own, stage, lds_lg, lds_tokens);
        else k_tile<G, true>(a, b, h, blk, len_k, ks, 0, tm, kpre, true, own, stage, lds_lg, lds_tokens);
        blk += 1;
        fold(tm);
    }
    while (blk < blk_end) {
        float tm[G], later[G][4];
        if (blk == keep_blk) k_tile<G, false>(a, b, h, blk, len_k, ks, 0, tm, kpre, false, later, stage, lds_lg, lds_tokens);
        else k_tile<G, true>(a, b, h, blk, len_k, ks, 0, tm, kpre, false, later, stage, lds_lg, lds_tokens);
        blk += 1;
        fold(tm);
    }
    if (lane == 0)
#pragma unroll
        for (int g = 0; g < G; ++g) wmax_s[g][wave] = wm[g];
    // The new token's logit: one lane per query head walks its fp16 row in channel order.  Wave 0 does it after
    // its own tile -- the wave that is done first and would otherwise wait at the barrier below.
    if (attend_new && tid < G) ks.new_logit[tid] = new_token_logit<G>(ks, tid);
    if (tid == 0 && a.k_new) {
        stores_done();   // ordered after the read of the length
        ticket = take_ticket(&a.flags[AKV_NFLAGS + b]);
    }
    // The batches of 8*KG V rows are dealt over the waves in contiguous, balanced ranges, like the K blocks (timed against
    // taking turns batch by batch: 1 % faster).  A wave that is done with its tiles has nothing to do until the mid step
    // has run: it fetches the HI bytes of its first batches now (they depend on nothing).  Not when the row that is
    // being appended lies among those rows -- its bytes are stored below.
    constexpr int KG = head_v_groups<G, NT>(), RB = 8 * KG, kHeadVPre = head_v_pre<G>();
    const int nbatch = (len + RB - 1) / RB;
    const int vb0 = (int)((long long)nbatch * wave_u / kWaves), vb1 = (int)((long long)nbatch * (wave_u + 1) / kWaves);
    const bool pre_ok = !(appended && len_old < (vb0 + kHeadVPre) * RB);   // false only where the new row lies in the rows fetched here
    u32x4_t pre[kHeadVPre][KG];
    v_prefetch_hi<KG, kHeadVPre>(a, b, h, vb0 * RB, RB, pre_ok ? len : 0, pre);
    if (appended && tid < kD) {   // the new token goes into the planes (the block's lines were just read: they are in L2), K_colmax follows
        store_token_rmw(const_cast<uint8_t*>(a.k_hi), const_cast<uint8_t*>(a.k_mid), const_cast<uint8_t*>(a.k_lo),
                        const_cast<uint8_t*>(a.v_hi), const_cast<uint8_t*>(a.v_mid), const_cast<uint8_t*>(a.v_lo), bh,
                        Ncap, len_old, tid, a.k_new + bh * kD, a.v_new + bh * kD, old_m, old_l);
        const_cast<uint16_t*>(a.colmax)[bh * kD + tid] = (uint16_t)colmax_used;
    }
    __syncthreads();   // also: every logit store and the new token's bytes have completed (same CU, same L2)
    if (tid < G) {
        float m = -INFINITY;
        if (attend_new) {   // after the barrier: the tile that covers position len_old has stored its vector
            m = ks.new_logit[tid];
            if (LDSLG) lds_lg[tid * lds_tokens + len_old] = m;
            if (!LDSLG || a.dbg.logits) a.logits[(size_t(b) * Hq + size_t(h) * G + tid) * Ncap + len_old] = m;
        }
        for (int w = 0; w < kWaves; ++w) m = fmaxf(m, wmax_s[tid][w]);
        ms.M[tid] = m;
    }
    __syncthreads();

    // ---- mid step -----------------------------------------------------------------------------------
    const bool own_ok = nblk <= kWaves;   // then wave w < nblk has walked exactly block w, four tokens per lane
    if (own_ok && attend_new && (len_old >> 2) == tid) {   // the new token's logit did not come from a tile
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if ((len_old & 3) == i) own[g][i] = ks.new_logit[g];
    }
    mid_step<G, NT>(a, b, h, len, ms, own, own_ok, lds_lg, lds_tokens);

    // ---- V side: each wave walks its range of batches of 8*KG rows -------------------------------------
    VRule vr;
    v_rule_setup(ms.ehat, a.guard_bits, a.force_level, vr);
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
    v_rows<G, KG, DEBUG, kHeadVPre, kHeadVPre>(a, b, h, vb0 * RB, RB, vb1 - vb0, len, vr, Mg, acc, z, pre, pre_ok, lds_lg, lds_tokens);
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

// bytes of LDS a head workgroup may spend on logits beside its static arrays (staging areas of the K tiles, mid step,
// reduction): 160 KB per compute unit, one workgroup of 1024 threads or two of 512
template <int NT> constexpr size_t head_lds_logit_budget() { return NT >= 1024 ? 48 * 1024 : 32 * 1024; }

static int head_lds_tokens(const akv_shape& s, int max_len) { return (std::min(max_len, s.Ncap) + kTB - 1) / kTB * kTB; }   // the K tiles write whole blocks

bool head_logits_in_lds(const akv_shape& s, int max_len)
{
    const int G = s.Hq / s.Hkv;
    const size_t bytes = size_t(G) * head_lds_tokens(s, max_len) * sizeof(float);
    return bytes <= (G == 1 ? head_lds_logit_budget<1024>() : head_lds_logit_budget<512>());
}

template <int G, int NT>
static hipError_t launch_head_g(const DecodeArgs& a, hipStream_t st)
{
    const dim3 grid(xcd_grid(size_t(a.s.B) * a.s.Hkv)), block(NT);
    const bool debug = a.dbg.needV || a.dbg.appliedV || a.stats;
    const int lds_tokens = head_lds_tokens(a.s, a.max_len);
    const size_t lds_bytes = size_t(G) * lds_tokens * sizeof(float);
    if (head_logits_in_lds(a.s, a.max_len)) {
        static bool raised[64] = {};   // per instantiation and device: allow the dynamic part beside the static arrays
        auto kd = head_kernel<G, NT, true, true>;
        auto kp = head_kernel<G, NT, false, true>;
        int dev = 0;
        if (hipError_t e = hipGetDevice(&dev)) return e;
        if (dev < 0 || dev >= 64 || !raised[dev]) {
            if (hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kd), hipFuncAttributeMaxDynamicSharedMemorySize, (int)head_lds_logit_budget<NT>())) return e;
            if (hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kp), hipFuncAttributeMaxDynamicSharedMemorySize, (int)head_lds_logit_budget<NT>())) return e;
            if (dev >= 0 && dev < 64) raised[dev] = true;
        }
        if (debug) hipLaunchKernelGGL(kd, grid, block, lds_bytes, st, a, lds_tokens);
        else hipLaunchKernelGGL(kp, grid, block, lds_bytes, st, a, lds_tokens);
    } else {
        if (debug) hipLaunchKernelGGL((head_kernel<G, NT, true, false>), grid, block, 0, st, a, 0);
        else hipLaunchKernelGGL((head_kernel<G, NT, false, false>), grid, block, 0, st, a, 0);
    }
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
