// Between the two streaming passes: global max logit, score exponents, approximate top-k, O_est and the
// result exponents Rule 2 aligns to.
// "Quantization of V-Cache": the scores differ by orders of magnitude, so the product of a few of the
// largest scores with their V rows estimates the result (O_est); an approximate top-k picks them.
#pragma once
#include "akv_common.h"

namespace akv {

constexpr int kMidMaxWaves = 16;

// LDS of the mid step (declared __shared__ by the kernel that runs it)
struct MidShared {
    float M[kMaxG];              // in: global max logit of every query head of the group (set by the caller)
    int ehat[kD];                // out: result exponent per channel, min over the group
    int cnt[kBuckets];
    int wlt[kMidMaxWaves], weq[kMidMaxWaves];
    int sel[AKV_MAX_TOPK];
    float phat[AKV_MAX_TOPK];
    uint16_t v[AKV_MAX_TOPK][kD];
    int J, fromcut;
};

// Run by one workgroup of NT threads for one (sequence b, KV head h) of len tokens, after every logit of the pair is
// visible to it and sm.M holds the global max logit of each query head; the G query heads of the group are
// handled one after another.  CROSS: the logits were written by other workgroups of the same kernel and are
// read at device scope.  Logits are walked 4*NT at a time (a float4 per thread); the selected V rows are
// fetched by all threads at once into LDS so that O_est costs one memory latency, then each channel runs its
// ordered FMA chain.  Results: a.M, a.Ehat (global, for a later kernel) and sm.ehat (LDS).
template <int G, int NT, bool CROSS>
__device__ __forceinline__ void mid_step(const DecodeArgs& a, int b, int h, int len, MidShared& sm)
{
    constexpr int kWaves = NT / 64;
    constexpr int kChunk = NT * 4;
    static_assert(kWaves <= kMidMaxWaves && NT >= kD, "workgroup size");
    int (&cnt_s)[kBuckets] = sm.cnt;
    int (&wlt_s)[kMidMaxWaves] = sm.wlt;
    int (&weq_s)[kMidMaxWaves] = sm.weq;
    int (&sel_s)[AKV_MAX_TOPK] = sm.sel;
    float (&phat_s)[AKV_MAX_TOPK] = sm.phat;
    uint16_t (&v_s)[AKV_MAX_TOPK][kD] = sm.v;
    int& J_s = sm.J;
    int& fromcut_s = sm.fromcut;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int Hkv = a.s.Hkv, Hq = a.s.Hq, Ncap = a.s.Ncap;
    const size_t bh = size_t(b) * Hkv + h;
    int ehat = 32767;   // min over the group of the result exponent of channel tid (tid < D)

    for (int g = 0; g < G; ++g) {
        const size_t hq = size_t(b) * Hq + size_t(h) * G + g;
        const __amdgpu_buffer_rsrc_t rs_lg = make_rsrc(a.logits + hq * Ncap, uint32_t(Ncap) * 4u);
        auto load4 = [&](int t0) -> float4 {   // Ncap % 256 == 0: the vector stays inside the row
            const u32x4_t w = CROSS ? __builtin_amdgcn_raw_buffer_load_b128(rs_lg, uint32_t(t0) * 4u, 0, kAuxSc1)
                                    : __builtin_amdgcn_raw_buffer_load_b128(rs_lg, uint32_t(t0) * 4u, 0, 0);
            return make_float4(bits_float(w.x), bits_float(w.y), bits_float(w.z), bits_float(w.w));
        };
        if (len == 0) {
            if (tid == 0) a.M[hq] = 0.0f;
            continue;
        }
        const float M = sm.M[g];
        if (tid < kBuckets) cnt_s[tid] = 0;
        __syncthreads();

        // ---- histogram of score exponents: bucket j = -a_t, 0..64 -------------------------------------
        for (int t0 = tid * 4; t0 < len; t0 += kChunk) {
            const float4 l4 = load4(t0);
            const float lv[4] = {l4.x, l4.y, l4.z, l4.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (t0 + i < len) {
                    const int at = score_a(score_x(lv[i], M, a.c));
                    atomicAdd(&cnt_s[-at], 1);
                    if (a.dbg.a) a.dbg.a[hq * Ncap + t0 + i] = (int8_t)at;
                }
            }
        }
        __syncthreads();
        const int kk = a.topk < len ? a.topk : len;
        if (tid == 0) {
            int J = 0, below = 0;   // below = tokens in buckets < J
            while (below + cnt_s[J] < kk) below += cnt_s[J++];
            J_s = J;
            fromcut_s = kk - below;
        }
        __syncthreads();
        const int J = J_s, fromcut = fromcut_s;

        // ---- ordered selection: every token above the cut bucket, the first `fromcut` of the cut bucket --
        int tot_lt = 0, tot_eq = 0;   // tokens of each kind before the current chunk (same in all threads)
        for (int c0 = 0; c0 < len; c0 += kChunk) {
            const int t0 = c0 + tid * 4;
            float x[4];
            int j[4];
            int c_lt = 0, c_eq = 0;
            if (t0 < len) {
                const float4 l4 = load4(t0);
                const float lv[4] = {l4.x, l4.y, l4.z, l4.w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    x[i] = score_x(lv[i], M, a.c);
                    j[i] = t0 + i < len ? -score_a(x[i]) : 1000;
                    c_lt += j[i] < J;
                    c_eq += j[i] == J;
                }
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    x[i] = 0.0f;
                    j[i] = 1000;
                }
            }
            int s_lt = c_lt, s_eq = c_eq;   // inclusive scan over the lanes of the wave
            for (int o = 1; o < 64; o <<= 1) {
                const int u_lt = __shfl_up(s_lt, o), u_eq = __shfl_up(s_eq, o);
                if (lane >= o) {
                    s_lt += u_lt;
                    s_eq += u_eq;
                }
            }
            if (lane == 63) {
                wlt_s[wave] = s_lt;
                weq_s[wave] = s_eq;
            }
            __syncthreads();
            int n_lt = tot_lt + s_lt - c_lt, n_eq = tot_eq + s_eq - c_eq;   // tokens of each kind before this thread's four
            int chunk_lt = 0, chunk_eq = 0;
            for (int w = 0; w < kWaves; ++w) {
                if (w < wave) {
                    n_lt += wlt_s[w];
                    n_eq += weq_s[w];
                }
                chunk_lt += wlt_s[w];
                chunk_eq += weq_s[w];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const bool is_lt = j[i] < J, is_eq = j[i] == J;
                if (is_lt || (is_eq && n_eq < fromcut)) {
                    const int pos = n_lt + (n_eq < fromcut ? n_eq : fromcut);
                    const float fl = floorf(x[i]);
                    const float f = x[i] - fl;
                    sel_s[pos] = t0 + i;
                    phat_s[pos] = ldexpf(1.0f + f, -j[i]);   // piecewise-linear 2^x with the exponent floored at -64
                }
                n_lt += is_lt;
                n_eq += is_eq;
            }
            tot_lt += chunk_lt;
            tot_eq += chunk_eq;
            __syncthreads();
            if (tot_lt + (tot_eq < fromcut ? tot_eq : fromcut) >= kk) break;   // uniform
        }
        __syncthreads();

        // ---- the selected rows at full 16 bits -> LDS (8 threads per row, all rows in flight together) ----
        for (int row = tid >> 3; row < kk; row += NT / 8) {
            const int cl = tid & 7;
            const size_t vrow = bh * Ncap + sel_s[row];
            const uint4 hi = *reinterpret_cast<const uint4*>(a.v_hi + vrow * kD + cl * 16);
            const uint2 mid = *reinterpret_cast<const uint2*>(a.v_mid + vrow * (kD / 2) + cl * 8);
            const uint2 lo = *reinterpret_cast<const uint2*>(a.v_lo + vrow * (kD / 2) + cl * 8);
            uint32_t pa[4], pb[4];
            assemble8(hi.x, hi.y, mid.x, lo.x, pa);
            assemble8(hi.z, hi.w, mid.y, lo.y, pb);
            uint16_t* dst = &v_s[row][cl * 16];
            const uint32_t pp[8] = {pa[0], pa[1], pa[2], pa[3], pb[0], pb[1], pb[2], pb[3]};
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {   // pairs (0,2),(1,3) then (4,6),(5,7) of each eight
                const uint32_t e = pp[2 * q4], o = pp[2 * q4 + 1];
                const int base = (q4 >> 1) * 8 + (q4 & 1) * 4;
                dst[base + 0] = (uint16_t)e;
                dst[base + 1] = (uint16_t)o;
                dst[base + 2] = (uint16_t)(e >> 16);
                dst[base + 3] = (uint16_t)(o >> 16);
            }
        }
        __syncthreads();

        // ---- O_est: ordered FMA chain per channel, result exponents ----------------------------------
        if (tid < kD) {
            const int d = tid;
            float acc = 0.0f;
            for (int i = 0; i < kk; ++i) acc = fmaf(phat_s[i], half_bits_to_float(v_s[i][d]), acc);
            const int E = float_exp_field(acc) - 127;
            ehat = E < ehat ? E : ehat;
            if (a.dbg.oest) a.dbg.oest[hq * kD + d] = acc;
        }
        if (a.dbg.sel && tid < a.topk) a.dbg.sel[hq * a.topk + tid] = tid < kk ? sel_s[tid] : -1;
        if (tid == 0) a.M[hq] = M;
        __syncthreads();
    }
    if (tid < kD) {
        sm.ehat[tid] = ehat;
        a.Ehat[bh * kD + tid] = ehat;
        if (a.dbg.Ehat) a.dbg.Ehat[bh * kD + tid] = (int16_t)ehat;
    }
    __syncthreads();
}

}  // namespace akv
