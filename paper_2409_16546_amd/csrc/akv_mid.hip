// Between the two streaming passes: global max logit, score exponents, approximate top-k, O_est and the
// result exponents Rule 2 aligns to.
// "Quantization of V-Cache": the scores differ by orders of magnitude, so the product of a few of the
// largest scores with their V rows estimates the result (O_est); an approximate top-k picks them.
#include "akv_common.h"

namespace akv {

constexpr int kMidThreads = 256;

// One workgroup per (sequence, KV head); the G query heads of the group are handled one after another.
template <int G>
__global__ __launch_bounds__(kMidThreads) void mid_kernel(DecodeArgs a)
{
    __shared__ int cnt_s[kBuckets];
    __shared__ float redf_s[kMidThreads / 64];
    __shared__ int wlt_s[kMidThreads / 64], weq_s[kMidThreads / 64];
    __shared__ int sel_s[AKV_MAX_TOPK];
    __shared__ float phat_s[AKV_MAX_TOPK];
    __shared__ int J_s, fromcut_s;

    const int h = blockIdx.x, b = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int Hkv = a.s.Hkv, Hq = a.s.Hq, Ncap = a.s.Ncap;
    const int len = min(a.lens[b], Ncap);
    const size_t bh = size_t(b) * Hkv + h;
    const int ntile = k_tiles(Ncap);
    int ehat = 32767;   // min over the group of the result exponent of channel tid (tid < D)

    for (int g = 0; g < G; ++g) {
        const size_t hq = size_t(b) * Hq + size_t(h) * G + g;
        const float* lg = a.logits + hq * Ncap;
        if (len == 0) {
            if (tid == 0) a.M[hq] = 0.0f;
            continue;
        }
        // ---- M = max_t l_t (exact, order-free) ------------------------------------------------------
        float m = -INFINITY;
        for (int i = tid; i < k_tiles(len); i += kMidThreads) m = fmaxf(m, a.tilemax[hq * ntile + i]);
        m = wave_max(m);
        if (tid < kBuckets) cnt_s[tid] = 0;
        if (lane == 0) redf_s[wave] = m;
        __syncthreads();
        float M = redf_s[0];
        for (int w = 1; w < kMidThreads / 64; ++w) M = fmaxf(M, redf_s[w]);

        // ---- histogram of score exponents: bucket j = -a_t, 0..64 -------------------------------------
        for (int t = tid; t < len; t += kMidThreads) {
            const int at = score_a(score_x(lg[t], M, a.c));
            atomicAdd(&cnt_s[-at], 1);
            if (a.dbg.a) a.dbg.a[hq * Ncap + t] = (int8_t)at;
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
        for (int c0 = 0; c0 < len; c0 += kMidThreads) {
            const int t = c0 + tid;
            float x = 0.0f;
            int j = 1000;
            if (t < len) {
                x = score_x(lg[t], M, a.c);
                j = -score_a(x);
            }
            const bool is_lt = j < J, is_eq = j == J;
            const uint64_t blt = __ballot(is_lt), beq = __ballot(is_eq);
            const uint64_t below_me = (uint64_t(1) << lane) - 1;
            if (lane == 0) {
                wlt_s[wave] = __popcll(blt);
                weq_s[wave] = __popcll(beq);
            }
            __syncthreads();
            int n_lt = tot_lt + __popcll(blt & below_me), n_eq = tot_eq + __popcll(beq & below_me);
            int chunk_lt = 0, chunk_eq = 0;
            for (int w = 0; w < kMidThreads / 64; ++w) {
                if (w < wave) {
                    n_lt += wlt_s[w];
                    n_eq += weq_s[w];
                }
                chunk_lt += wlt_s[w];
                chunk_eq += weq_s[w];
            }
            if (is_lt || (is_eq && n_eq < fromcut)) {
                const int pos = n_lt + (n_eq < fromcut ? n_eq : fromcut);
                const float fl = floorf(x);
                const float f = x - fl;
                sel_s[pos] = t;
                phat_s[pos] = ldexpf(1.0f + f, -j);   // piecewise-linear 2^x with the exponent floored at -64
            }
            tot_lt += chunk_lt;
            tot_eq += chunk_eq;
            __syncthreads();
            if (tot_lt + (tot_eq < fromcut ? tot_eq : fromcut) >= kk) break;   // uniform
        }
        __syncthreads();

        // ---- O_est over the selected rows at full 16 bits, result exponents --------------------------
        if (tid < kD) {
            const int d = tid;
            float acc = 0.0f;
            for (int i = 0; i < kk; ++i) {
                const size_t row = bh * Ncap + sel_s[i];
                const uint32_t hi = a.v_hi[row * kD + d];
                const uint32_t mb = a.v_mid[row * (kD / 2) + d / 2], lb = a.v_lo[row * (kD / 2) + d / 2];
                const uint32_t mn = (d & 1) ? (mb >> 4) : (mb & 15u), ln = (d & 1) ? (lb >> 4) : (lb & 15u);
                acc = fmaf(phat_s[i], half_bits_to_float((hi << 8) | (mn << 4) | ln), acc);
            }
            const int E = float_exp_field(acc) - 127;
            ehat = E < ehat ? E : ehat;
            if (a.dbg.oest) a.dbg.oest[hq * kD + d] = acc;
        }
        if (a.dbg.sel && tid < a.topk) a.dbg.sel[hq * a.topk + tid] = tid < kk ? sel_s[tid] : -1;
        if (tid == 0) a.M[hq] = M;
        __syncthreads();
    }
    if (tid < kD) {
        a.Ehat[bh * kD + tid] = ehat;
        if (a.dbg.Ehat) a.dbg.Ehat[bh * kD + tid] = (int16_t)ehat;
    }
}

hipError_t launch_mid(const DecodeArgs& a, hipStream_t st)
{
    const int G = a.s.Hq / a.s.Hkv;
    const dim3 grid(a.s.Hkv, a.s.B), block(kMidThreads);
    switch (G) {
        case 1: hipLaunchKernelGGL(mid_kernel<1>, grid, block, 0, st, a); break;
        case 2: hipLaunchKernelGGL(mid_kernel<2>, grid, block, 0, st, a); break;
        case 4: hipLaunchKernelGGL(mid_kernel<4>, grid, block, 0, st, a); break;
        case 8: hipLaunchKernelGGL(mid_kernel<8>, grid, block, 0, st, a); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace akv
