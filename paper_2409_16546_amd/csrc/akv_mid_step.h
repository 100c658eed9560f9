// Between the two streaming passes: global max logit, score exponents, approximate top-k, O_est and the
// result exponents Rule 2 aligns to.
// "Quantization of V-Cache": the scores differ by orders of magnitude, so the product of a few of the
// largest scores with their V rows estimates the result (O_est); an approximate top-k picks them.
#pragma once
#include "akv_common.h"

namespace akv {

constexpr int kMidMaxWaves = 16;
constexpr int kMidSets = 4;   // selections that can be held at once

// LDS of the mid step (declared __shared__ by the kernel that runs it)
struct MidShared {
    float M[kMaxG];              // in: global max logit of every query head of the group (set by the caller)
    int ehat[kD];                // out: result exponent per channel, min over the group
    int cnt[kBuckets];           // histogram of score exponents (several chunks of tokens per thread)
    int cntw[kMidMaxWaves][kBuckets + 1];   // ... per wave (one chunk: every thread owns four tokens)
    int wlt[kMidMaxWaves], weq[kMidMaxWaves];
    int sel[kMidSets][AKV_MAX_TOPK];                  // selected tokens, ascending (several query heads at a time
    alignas(16) float phat[kMidSets][AKV_MAX_TOPK];   // in the token-split kernel, else set 0)
    int selj[kMidSets][AKV_MAX_TOPK];                 // their buckets
    alignas(16) uint32_t v2[AKV_MAX_TOPK / 2][kD];   // fp16 bits of the selected V rows: rows 2i (low half) and 2i+1 of channel d
};

// position pos of a selected token: its index and piecewise-linear weight go to LDS
__device__ __forceinline__ void mid_emit(MidShared& sm, int set, int pos, int t, float x, int j)
{
    const float fl = floorf(x);
    const float f = x - fl;
    sm.sel[set][pos] = t;
    sm.selj[set][pos] = j;
    sm.phat[set][pos] = ldexpf(1.0f + f, -j);   // 2^x with a linear mantissa, the exponent floored at -64
}

// One token per lane into a histogram in LDS (buckets 0..64; a token that does not count has j > 64; called by all
// lanes of a wave).  The floor bucket 64 takes every weight below 2^-64 -- most tokens of a peaked softmax -- and an
// LDS atomic whose lanes all hit one address costs a cycle per lane of the one LDS unit the waves of a compute unit
// share: that bucket is counted with a ballot (n64, wave-uniform, handed to mid_hist_flush at the end), only the
// others with atomics.
__device__ __forceinline__ void mid_hist_add(int* hist, int j, int& n64)
{
    n64 += __builtin_popcountll(__ballot(j == 64));
    if (j < 64) atomicAdd(&hist[j], 1);
}
__device__ __forceinline__ void mid_hist_flush(int* hist, int n64)
{
    if ((threadIdx.x & 63) == 0 && n64 > 0) atomicAdd(&hist[64], n64);
}

// The cut from bucket totals (lane l of a full wave holds the total of bucket l; bucket 64 can only be the cut if
// none before it is): first bucket J where the running count reaches kk, and the number of tokens in buckets below it.
__device__ __forceinline__ void mid_find_cut(int c, int kk, int& J, int& below)
{
    const int incl = wave_scan_add(c);
    const uint64_t reached = __ballot(incl >= kk);
    J = reached ? __builtin_ctzll(reached) : 64;
    below = J == 0 ? 0 : wave_read(incl, J - 1);
}

// tokens of each kind in lower lanes of the wave (token order = lane, then i), and in the whole wave
__device__ __forceinline__ void mid_wave_order(const int (&j)[4], int J, int& n_lt, int& n_eq, int& w_lt, int& w_eq)
{
    n_lt = n_eq = w_lt = w_eq = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint64_t b_lt = __ballot(j[i] < J), b_eq = __ballot(j[i] == J);
        n_lt += __builtin_amdgcn_mbcnt_hi((uint32_t)(b_lt >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)b_lt, 0));
        n_eq += __builtin_amdgcn_mbcnt_hi((uint32_t)(b_eq >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)b_eq, 0));
        w_lt += __builtin_popcountll(b_lt);
        w_eq += __builtin_popcountll(b_eq);
    }
}

// The approximate top-kk of one chunk of 4*NT tokens in token order (thread -> tokens t0 .. t0+3 with score x and
// bucket j, 1000 for a token that does not count), called by all NT threads; sm.cntw must be zero on entry (and a
// barrier must lie between the zeroing and this call).  Per-wave histograms (LDS atomics) give every wave the cut
// bucket and the number of selected tokens in the waves before it with one barrier; ballots order the tokens
// inside a wave.  The selection goes to set `set` of sm; returns the cut bucket.
template <int NT>
__device__ __forceinline__ int mid_select_chunk(MidShared& sm, int set, const float (&x)[4], const int (&j)[4], int t0, int kk)
{
    constexpr int kWaves = NT / 64;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int n64 = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) mid_hist_add(&sm.cntw[wave][0], j[i], n64);
    mid_hist_flush(&sm.cntw[wave][0], n64);
    __syncthreads();
    int tot = 0, before = 0;   // bucket `lane`: all waves / the waves before this one
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        const int c = sm.cntw[w][lane];
        tot += c;
        before += w < wave ? c : 0;
    }
    int J, below;
    mid_find_cut(tot, kk, J, below);
    const int fromcut = kk - below;
    // selected-for-sure tokens in earlier waves: buckets < J; tokens of the cut bucket in earlier waves
    const int base_lt = wave_read(wave_scan_add(lane < J ? before : 0), 63);
    int base_eq;
    if (J < 64) {
        base_eq = wave_read(before, J);
    } else {
        base_eq = 0;
        for (int w = 0; w < wave; ++w) base_eq += sm.cntw[w][64];
    }
    int n_lt, n_eq, w_lt, w_eq;
    mid_wave_order(j, J, n_lt, n_eq, w_lt, w_eq);
    n_lt += base_lt;
    n_eq += base_eq;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const bool is_lt = j[i] < J, is_eq = j[i] == J;
        if (is_lt || (is_eq && n_eq < fromcut)) mid_emit(sm, set, n_lt + (n_eq < fromcut ? n_eq : fromcut), t0 + i, x[i], j[i]);
        n_lt += is_lt;
        n_eq += is_eq;
    }
    return J;
}

// O_est of one query head from the kk selected tokens in sm.sel[set] / sm.phat[set] (all threads of the workgroup;
// contains barriers, the last one after the LDS rows have been read): the selected V rows at full 16 bits go to LDS (8 threads per row, all rows in flight together, so
// that this costs one memory latency), then each channel runs its ordered FMA chain from operands fetched 16 rows
// at a time.  ehat (thread d < 128: channel d) is lowered to the exponent of the result.
// The selected V rows of one query head, 16 bits of every element, as they come from memory: thread -> (row
// tid / 8 + p * NT / 8 of the selection, 16-channel slice tid % 8)
template <int NT>
struct OestRows {
    static constexpr int kPasses = (AKV_MAX_TOPK + NT / 8 - 1) / (NT / 8);
    uint4 hi[kPasses];
    uint2 mid[kPasses], lo[kPasses];
};
// issue the loads of the rows sm.sel[set][0 .. kk-1] (nothing waits for them here: a caller with several query
// heads asks for all of them before it uses the first)
template <int NT>
__device__ __forceinline__ void mid_oest_fetch(const DecodeArgs& a, size_t bh, int kk, const MidShared& sm, int set, OestRows<NT>& R)
{
    const int tid = threadIdx.x, cl = tid & 7;
#pragma unroll
    for (int p = 0; p < OestRows<NT>::kPasses; ++p) {
        const int row = (tid >> 3) + p * (NT / 8);
        if (row < kk) {
            const size_t vrow = bh * a.s.Ncap + sm.sel[set][row];
            R.hi[p] = *reinterpret_cast<const uint4*>(a.v_hi + vrow * kD + cl * 16);
            R.mid[p] = *reinterpret_cast<const uint2*>(a.v_mid + vrow * (kD / 2) + cl * 8);
            R.lo[p] = *reinterpret_cast<const uint2*>(a.v_lo + vrow * (kD / 2) + cl * 8);
        }
    }
}
// rows -> LDS (two rows per word), then each channel runs its ordered FMA chain; ends with a barrier
template <int NT>
__device__ __forceinline__ void mid_oest_finish(const DecodeArgs& a, size_t hq, int kk, MidShared& sm, int set, const OestRows<NT>& R,
                                                int& ehat)
{
    const int tid = threadIdx.x, cl = tid & 7;
#pragma unroll
    for (int p = 0; p < OestRows<NT>::kPasses; ++p) {
        const int row = (tid >> 3) + p * (NT / 8);
        if (row < kk) {
            uint32_t pa[4], pb[4];
            assemble8(R.hi[p].x, R.hi[p].y, R.mid[p].x, R.lo[p].x, pa);
            assemble8(R.hi[p].z, R.hi[p].w, R.mid[p].y, R.lo[p].y, pb);
            uint16_t* dst = reinterpret_cast<uint16_t*>(&sm.v2[row >> 1][cl * 16]) + (row & 1);   // element stride: 2 halves
            const uint32_t pp[8] = {pa[0], pa[1], pa[2], pa[3], pb[0], pb[1], pb[2], pb[3]};
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {   // pairs (0,2),(1,3) then (4,6),(5,7) of each eight
                const uint32_t e = pp[2 * q4], o = pp[2 * q4 + 1];
                const int base = (q4 >> 1) * 8 + (q4 & 1) * 4;
                dst[2 * (base + 0)] = (uint16_t)e;
                dst[2 * (base + 1)] = (uint16_t)o;
                dst[2 * (base + 2)] = (uint16_t)(e >> 16);
                dst[2 * (base + 3)] = (uint16_t)(o >> 16);
            }
        }
    }
    __syncthreads();
    if (tid < kD) {
        const int d = tid;
        float acc = 0.0f;
        for (int i0 = 0; i0 < kk; i0 += 16) {   // the additions stay in selection order
            float pv[16];
            uint32_t vv[8];
#pragma unroll
            for (int i = 0; i < 16; i += 4) {
                const float4 p4 = *reinterpret_cast<const float4*>(&sm.phat[set][i0 + i]);
                pv[i] = p4.x; pv[i + 1] = p4.y; pv[i + 2] = p4.z; pv[i + 3] = p4.w;
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) vv[i] = sm.v2[(i0 >> 1) + i][d];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                if (i0 + 2 * i < kk) acc = fmaf(pv[2 * i], lo_half(vv[i]), acc);
                if (i0 + 2 * i + 1 < kk) acc = fmaf(pv[2 * i + 1], hi_half(vv[i]), acc);
            }
        }
        const int E = float_exp_field(acc) - 127;
        ehat = E < ehat ? E : ehat;
        if (a.dbg.oest) a.dbg.oest[hq * kD + d] = acc;
    }
    if (a.dbg.sel && tid < a.topk) a.dbg.sel[hq * a.topk + tid] = tid < kk ? sm.sel[set][tid] : -1;
    __syncthreads();
}
template <int NT>
__device__ __forceinline__ void mid_oest(const DecodeArgs& a, size_t bh, size_t hq, int kk, MidShared& sm, int set, int& ehat)
{
    OestRows<NT> R;
    mid_oest_fetch<NT>(a, bh, kk, sm, set, R);
    mid_oest_finish<NT>(a, hq, kk, sm, set, R, ehat);
}

// Run by one workgroup of NT threads for one (sequence b, KV head h) of len tokens, after every logit of the pair is
// visible to it and sm.M holds the global max logit of each query head; the G query heads of the group are
// handled one after another.
// use_own: own[g][i] is the logit of token 4*tid + i of query head g (the caller still has them in registers);
// only used when the sequence fits one chunk of 4*NT tokens.
// Token order is (thread, i) inside a chunk of 4*NT tokens, chunks ascending.  One chunk (the common case):
// per-wave histograms give every wave the cut bucket and the number of selected tokens in the waves before it
// without a second barrier; ballots order the tokens inside the wave.  The selected V rows are fetched by all
// threads at once into LDS so that O_est costs one memory latency, then each channel runs its ordered FMA chain
// from operands fetched up front.  Results: a.M, a.Ehat (global, for a later kernel) and sm.ehat (LDS).
// lds_lg / lds_stride: the logits in LDS as k_tile left them, or NULL (they are read from a.logits).
template <int G, int NT>
__device__ __forceinline__ void mid_step(const DecodeArgs& a, int b, int h, int len, MidShared& sm,
                                         const float (&own)[G][4], bool use_own, const float* lds_lg = nullptr,
                                         int lds_stride = 0)
{
    constexpr int kWaves = NT / 64;
    constexpr int kChunk = NT * 4;
    static_assert(kWaves <= kMidMaxWaves && NT >= kD, "workgroup size");
    int (&cnt_s)[kBuckets] = sm.cnt;
    int (&wlt_s)[kMidMaxWaves] = sm.wlt;
    int (&weq_s)[kMidMaxWaves] = sm.weq;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int Hkv = a.s.Hkv, Hq = a.s.Hq, Ncap = a.s.Ncap;
    const size_t bh = size_t(b) * Hkv + h;
    int ehat = 32767;   // min over the group of the result exponent of channel tid (tid < D)
    const bool one_chunk = len <= kChunk;   // uniform

    for (int g = 0; g < G; ++g) {
        const size_t hq = size_t(b) * Hq + size_t(h) * G + g;
        const __amdgpu_buffer_rsrc_t rs_lg = make_rsrc(a.logits + hq * Ncap, uint32_t(Ncap) * 4u);
        auto load4 = [&](int t0) -> float4 {   // Ncap % 256 == 0: the vector stays inside the row
            if (lds_lg) return *reinterpret_cast<const float4*>(lds_lg + g * lds_stride + t0);
            const u32x4_t w = __builtin_amdgcn_raw_buffer_load_b128(rs_lg, uint32_t(t0) * 4u, 0, 0);
            return make_float4(bits_float(w.x), bits_float(w.y), bits_float(w.z), bits_float(w.w));
        };
        if (len == 0) {
            if (tid == 0) a.M[hq] = 0.0f;
            continue;
        }
        const float M = sm.M[g];
        const int kk = a.topk < len ? a.topk : len;
        // score exponents of four tokens: x, and the bucket j = -a_t (1000 for tokens at or past len)
        auto score4 = [&](int t0, const float (&lv)[4], float (&x)[4], int (&j)[4]) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                x[i] = score_x(lv[i], M, a.c);
                j[i] = t0 + i < len ? -score_a(x[i]) : 1000;
            }
        };
        auto load_score4 = [&](int t0, float (&x)[4], int (&j)[4]) {
            float lv[4] = {0.0f, 0.0f, 0.0f, 0.0f};
            if (t0 < len) {
                const float4 l4 = load4(t0);
                lv[0] = l4.x; lv[1] = l4.y; lv[2] = l4.z; lv[3] = l4.w;
            }
            score4(t0, lv, x, j);
        };
        if (one_chunk) {
            // ---- per-wave histograms of score exponents: bucket j = -a_t, 0..64 -------------------------
            for (int idx = tid; idx < kWaves * (kBuckets + 1); idx += NT) (&sm.cntw[0][0])[idx] = 0;
            float x[4];
            int j[4];
            const int t0 = tid * 4;
            if (use_own) {
                float lv[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int gg = 0; gg < G; ++gg)   // static indices keep the caller's array in registers
#pragma unroll
                    for (int i = 0; i < 4; ++i) lv[i] = gg == g ? own[gg][i] : lv[i];
                score4(t0, lv, x, j);
            } else {
                load_score4(t0, x, j);
            }
            __syncthreads();
            if (a.dbg.a) {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (j[i] <= 64) a.dbg.a[hq * Ncap + t0 + i] = (int8_t)(-j[i]);
            }
            mid_select_chunk<NT>(sm, 0, x, j, t0, kk);
        } else {
            // ---- histogram of score exponents over all chunks -----------------------------------------
            if (tid < kBuckets) cnt_s[tid] = 0;
            __syncthreads();
            int n64 = 0;
            for (int c0 = 0; c0 < len; c0 += kChunk) {   // uniform trip count: the ballots below need whole waves
                const int t0 = c0 + tid * 4;
                float x[4];
                int j[4] = {1000, 1000, 1000, 1000};
                if (t0 < len) load_score4(t0, x, j);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    mid_hist_add(cnt_s, j[i], n64);
                    if (j[i] <= 64 && a.dbg.a) a.dbg.a[hq * Ncap + t0 + i] = (int8_t)(-j[i]);
                }
            }
            mid_hist_flush(cnt_s, n64);
            __syncthreads();
            int J, below;
            mid_find_cut(cnt_s[lane], kk, J, below);
            const int fromcut = kk - below;
            // ---- ordered selection, chunk by chunk --------------------------------------------------------
            int tot_lt = 0, tot_eq = 0;   // tokens of each kind before the current chunk (same in all threads)
            for (int c0 = 0; c0 < len; c0 += kChunk) {
                const int t0 = c0 + tid * 4;
                float x[4];
                int j[4];
                load_score4(t0, x, j);
                int n_lt, n_eq, w_lt, w_eq;
                mid_wave_order(j, J, n_lt, n_eq, w_lt, w_eq);
                if (lane == 0) {
                    wlt_s[wave] = w_lt;
                    weq_s[wave] = w_eq;
                }
                __syncthreads();
                n_lt += tot_lt;
                n_eq += tot_eq;
                int chunk_lt = 0, chunk_eq = 0;
#pragma unroll
                for (int w = 0; w < kWaves; ++w) {
                    const int a_lt = wlt_s[w], a_eq = weq_s[w];
                    if (w < wave) {
                        n_lt += a_lt;
                        n_eq += a_eq;
                    }
                    chunk_lt += a_lt;
                    chunk_eq += a_eq;
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const bool is_lt = j[i] < J, is_eq = j[i] == J;
                    if (is_lt || (is_eq && n_eq < fromcut)) mid_emit(sm, 0, n_lt + (n_eq < fromcut ? n_eq : fromcut), t0 + i, x[i], j[i]);
                    n_lt += is_lt;
                    n_eq += is_eq;
                }
                tot_lt += chunk_lt;
                tot_eq += chunk_eq;
                __syncthreads();
                if (tot_lt + (tot_eq < fromcut ? tot_eq : fromcut) >= kk) break;   // uniform
            }
        }
        __syncthreads();

        // ---- O_est from the selected rows, result exponents -------------------------------------------
        mid_oest<NT>(a, bh, hq, kk, sm, 0, ehat);
        if (tid == 0) a.M[hq] = M;
    }
    if (tid < kD) {
        sm.ehat[tid] = ehat;
        a.Ehat[bh * kD + tid] = ehat;
        if (a.dbg.Ehat) a.dbg.Ehat[bh * kD + tid] = (int16_t)ehat;
    }
    __syncthreads();
}

}  // namespace akv
