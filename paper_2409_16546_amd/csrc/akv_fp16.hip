// The unquantised yardstick: decode attention on plain fp16 K, V [B][Hkv][Ncap][D]
// ("Runtime of AlignedKV": S = QK^T/sqrt(128), softmax, O = SV on 16-bit data).
// Same streaming design as the plane kernels (16-byte coalesced loads straight into registers, wave
// shuffles for the reductions, token-axis splits combined at the end), but K and V of a chunk are read in
// one kernel with a chunk-local softmax (split-KV), since nothing has to be decided between the passes.
#include <type_traits>

#include "akv_common.h"

namespace akv {

// 16 bytes with the non-temporal hint (the token-split kernels stream K and V once per step, as the aligned ones do)
__device__ __forceinline__ uint4 load16_nt(const uint16_t* p)
{
    const u32x4_t w = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
    return make_uint4(w.x, w.y, w.z, w.w);
}

constexpr int kFChunk = 512;   // tokens per workgroup
constexpr int kFWaves = 4;

inline int f_splits(int ntok) { return (ntok + kFChunk - 1) / kFChunk; }

size_t fp16_workspace_bytes(const akv_shape& s)
{
    const size_t bhq = size_t(s.B) * s.Hq, ns = f_splits(s.Ncap);
    return align256(bhq * ns * kD * sizeof(float)) + 2 * align256(bhq * ns * sizeof(float)) +
           align256(bhq * size_t(s.Ncap) * sizeof(float));   // split partials, then the logits of the head-per-workgroup variant
}

struct F16Args {
    akv_shape s;
    const uint16_t *k, *v, *q;
    const int32_t* lens;
    void* out;
    float c;   // scale * log2(e)
    int out_dtype, nsplit, max_len;
    float *partO, *partM, *partZ;
};

__device__ __forceinline__ void unpack8h(const uint4& w, float (&f)[8])
{
    f[0] = lo_half(w.x); f[1] = hi_half(w.x); f[2] = lo_half(w.y); f[3] = hi_half(w.y);
    f[4] = lo_half(w.z); f[5] = hi_half(w.z); f[6] = lo_half(w.w); f[7] = hi_half(w.w);
}

// Workgroup = 4 waves, one (sequence, KV head, 512-token chunk).  A token row is 256 B = 16 lanes x 16 B;
// a wave reads 4 rows per step.  Phase 1: logits of the chunk into LDS (16-lane shuffle reduction).
// Phase 2: chunk max, p = 2^((l - m) c), Z and O accumulated per lane, reduced over rows and waves.
template <int G>
__global__ __launch_bounds__(64 * kFWaves) void fp16_kernel(F16Args a)
{
    __shared__ float l_s[G][kFChunk];
    __shared__ float red_s[kFWaves][G][kD + 1];
    __shared__ float max_s[kFWaves][G];

    const int h = blockIdx.y, b = blockIdx.z, split = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = lane >> 4, cl = lane & 15;            // row within the wave's group of 4, channels 8*cl..8*cl+7
    const int Hkv = a.s.Hkv, Hq = a.s.Hq, Ncap = a.s.Ncap;
    const int len = min(min(a.lens[b], Ncap), a.max_len);
    const int c0 = split * kFChunk;
    if (c0 >= len) return;
    const size_t bh = size_t(b) * Hkv + h;

    float qf[G][8];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const uint4 w = *reinterpret_cast<const uint4*>(a.q + (size_t(b) * Hq + size_t(h) * G + g) * kD + cl * 8);
        unpack8h(w, qf[g]);
    }

    // ---- phase 1: logits ---------------------------------------------------------------------------
    float mloc[G];
#pragma unroll
    for (int g = 0; g < G; ++g) mloc[g] = -INFINITY;
    for (int it = 0; it < kFChunk / (4 * kFWaves); ++it) {
        const int tl = it * (4 * kFWaves) + wave * 4 + r, t = c0 + tl;
        const bool valid = t < len;
        uint4 w = make_uint4(0, 0, 0, 0);
        if (valid) w = load16_nt(a.k + (bh * Ncap + t) * kD + cl * 8);
        float kf[8];
        unpack8h(w, kf);
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float s = 0.0f;
#pragma unroll
            for (int i = 0; i < 8; ++i) s = fmaf(qf[g][i], kf[i], s);
            for (int o = 1; o < 16; o <<= 1) s += __shfl_xor(s, o);
            if (valid) mloc[g] = fmaxf(mloc[g], s);
            if (cl == 0) l_s[g][tl] = s;
        }
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const float m = wave_max(mloc[g]);
        if (lane == 0) max_s[wave][g] = m;
    }
    __syncthreads();
    float mg[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        mg[g] = max_s[0][g];
        for (int w = 1; w < kFWaves; ++w) mg[g] = fmaxf(mg[g], max_s[w][g]);
    }

    // ---- phase 2: weights and O ---------------------------------------------------------------------
    float acc[G][8], z[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        z[g] = 0.0f;
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[g][i] = 0.0f;
    }
    for (int it = 0; it < kFChunk / (4 * kFWaves); ++it) {
        const int tl = it * (4 * kFWaves) + wave * 4 + r, t = c0 + tl;
        const bool valid = t < len;
        uint4 w = make_uint4(0, 0, 0, 0);
        if (valid) w = load16_nt(a.v + (bh * Ncap + t) * kD + cl * 8);
        float vf[8];
        unpack8h(w, vf);
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float p = valid ? __builtin_amdgcn_exp2f((l_s[g][tl] - mg[g]) * a.c) : 0.0f;
            z[g] += p;
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[g][i] = fmaf(p, vf[i], acc[g][i]);
        }
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
        for (int o = 16; o < 64; o <<= 1) {
            z[g] += __shfl_xor(z[g], o);
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[g][i] += __shfl_xor(acc[g][i], o);
        }
        if (r == 0) {
#pragma unroll
            for (int i = 0; i < 8; ++i) red_s[wave][g][cl * 8 + i] = acc[g][i];
            if (cl == 0) red_s[wave][g][kD] = z[g];
        }
    }
    __syncthreads();
    for (int idx = tid; idx < G * (kD + 1); idx += 64 * kFWaves) {
        const int g = idx / (kD + 1), d = idx % (kD + 1);
        float s = 0.0f;
#pragma unroll
        for (int w = 0; w < kFWaves; ++w) s += red_s[w][g][d];
        const size_t hq = size_t(b) * Hq + size_t(h) * G + g;
        if (d < kD) a.partO[(hq * a.nsplit + split) * kD + d] = s;
        else {
            a.partZ[hq * a.nsplit + split] = s;
            a.partM[hq * a.nsplit + split] = mg[g];
        }
    }
}

// merge the splits: rescale each to the global max
__global__ __launch_bounds__(kD) void fp16_combine_kernel(F16Args a)
{
    const int hq_i = blockIdx.x, b = blockIdx.y, d = threadIdx.x;
    const int len = min(min(a.lens[b], a.s.Ncap), a.max_len);
    const size_t hq = size_t(b) * a.s.Hq + hq_i;
    const int used = (len + kFChunk - 1) / kFChunk;
    float M = -INFINITY;
    for (int s = 0; s < used; ++s) M = fmaxf(M, a.partM[hq * a.nsplit + s]);
    float o = 0.0f, zsum = 0.0f;
    for (int s = 0; s < used; ++s) {
        const float w = __builtin_amdgcn_exp2f((a.partM[hq * a.nsplit + s] - M) * a.c);
        o = fmaf(w, a.partO[(hq * a.nsplit + s) * kD + d], o);
        zsum = fmaf(w, a.partZ[hq * a.nsplit + s], zsum);
    }
    const float res = used > 0 ? o / zsum : 0.0f;
    if (a.out_dtype == 0) reinterpret_cast<float*>(a.out)[hq * kD + d] = res;
    else reinterpret_cast<_Float16*>(a.out)[hq * kD + d] = (_Float16)res;
}

// Head-per-workgroup variant (the design of the plane kernels' main path): one workgroup of 1024 threads does
// the whole (sequence, KV head): logits of all tokens (kept in the workspace), their maximum, then weights and
// O.  A wave takes a contiguous range of the batches of 32 rows; the 8 row loads of the next batch are in flight while the
// current batch is reduced.
template <int G, int NT>
__global__ __launch_bounds__(NT) void fp16_head_kernel(F16Args a, float* __restrict__ logits)
{
    constexpr int kWaves = NT / 64;
    constexpr int kLoads = 8;   // 4 rows each
    __shared__ float max_s[kWaves][G];
    __shared__ float red_s[kWaves][G][kD + 1];

    const int Hkv = a.s.Hkv, Hq = a.s.Hq, Ncap = a.s.Ncap;
    const int pair = xcd_work_index(blockIdx.x, gridDim.x);   // an XCD takes consecutive heads
    if (pair >= a.s.B * Hkv) return;
    const int h = pair % Hkv, b = pair / Hkv;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = lane >> 4, cl = lane & 15;
    const int len = min(min(a.lens[b], Ncap), a.max_len);
    if (len == 0) {
        for (int idx = tid; idx < G * kD; idx += NT) {
            const size_t o = (size_t(b) * Hq + size_t(h) * G) * kD + idx;
            if (a.out_dtype == 0) reinterpret_cast<float*>(a.out)[o] = 0.0f;
            else reinterpret_cast<_Float16*>(a.out)[o] = (_Float16)0.0f;
        }
        return;
    }
    const size_t bh = size_t(b) * Hkv + h;
    const __amdgpu_buffer_rsrc_t rs_k = make_rsrc(a.k + bh * Ncap * kD, uint32_t(Ncap) * kD * 2u);
    const __amdgpu_buffer_rsrc_t rs_v = make_rsrc(a.v + bh * Ncap * kD, uint32_t(Ncap) * kD * 2u);
    float* lg[G];
    float qf[G][8];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const size_t hq = size_t(b) * Hq + size_t(h) * G + g;
        lg[g] = logits + hq * Ncap;
        const uint4 w = *reinterpret_cast<const uint4*>(a.q + hq * kD + cl * 8);
        unpack8h(w, qf[g]);
    }
    const int nbatch = (len + 31) / 32;
    // each wave walks a contiguous, balanced range of the batches, as in the aligned kernel of this shape
    const int bt0 = (int)((long long)nbatch * wave / kWaves), bt1 = (int)((long long)nbatch * (wave + 1) / kWaves);
    // the same cache hints as the aligned kernels of this shape: K non-temporal, V not
    auto load_batch = [&](const __amdgpu_buffer_rsrc_t& rs, int bt, u32x4_t (&w)[kLoads], auto nt) {
#pragma unroll
        for (int j = 0; j < kLoads; ++j) {
            const int t = bt * 32 + j * 4 + r;
            const uint32_t off = (bt < bt1 && t < len) ? uint32_t(t) * (kD * 2) + cl * 16 : kSkip;
            w[j] = decltype(nt)::value ? buf_load_b128_nt(rs, off) : buf_load_b128(rs, off);
        }
    };
    constexpr std::true_type kNt{};
    constexpr std::false_type kKeep{};

    // ---- phase 1: logits and their maximum ---------------------------------------------------------
    float mloc[G];
#pragma unroll
    for (int g = 0; g < G; ++g) mloc[g] = -INFINITY;
    u32x4_t wc[kLoads], wn[kLoads];
    load_batch(rs_k, bt0, wc, kNt);
#pragma unroll 1
    for (int bt = bt0; bt < bt1; ++bt) {
        load_batch(rs_k, bt + 1, wn, kNt);
#pragma unroll
        for (int j = 0; j < kLoads; ++j) {
            const int t = bt * 32 + j * 4 + r;
            float kf[8];
            unpack8h(make_uint4(wc[j].x, wc[j].y, wc[j].z, wc[j].w), kf);
#pragma unroll
            for (int g = 0; g < G; ++g) {
                float s = 0.0f;
#pragma unroll
                for (int i = 0; i < 8; ++i) s = fmaf(qf[g][i], kf[i], s);
                for (int o = 1; o < 16; o <<= 1) s += __shfl_xor(s, o);
                if (t < len) {
                    mloc[g] = fmaxf(mloc[g], s);
                    if (cl == 0) lg[g][t] = s;
                }
            }
        }
#pragma unroll
        for (int j = 0; j < kLoads; ++j) wc[j] = wn[j];
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const float m = wave_max(mloc[g]);
        if (lane == 0) max_s[wave][g] = m;
    }
    __syncthreads();   // also: every logit store of the workgroup has completed
    float mg[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        mg[g] = max_s[0][g];
        for (int w = 1; w < kWaves; ++w) mg[g] = fmaxf(mg[g], max_s[w][g]);
    }

    // ---- phase 2: weights and O -----------------------------------------------------------------------
    float acc[G][8], z[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        z[g] = 0.0f;
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[g][i] = 0.0f;
    }
    load_batch(rs_v, bt0, wc, kKeep);
#pragma unroll 1
    for (int bt = bt0; bt < bt1; ++bt) {
        load_batch(rs_v, bt + 1, wn, kKeep);
#pragma unroll
        for (int j = 0; j < kLoads; ++j) {
            const int t = bt * 32 + j * 4 + r;
            float vf[8];
            unpack8h(make_uint4(wc[j].x, wc[j].y, wc[j].z, wc[j].w), vf);
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const float p = t < len ? __builtin_amdgcn_exp2f((lg[g][t < len ? t : 0] - mg[g]) * a.c) : 0.0f;
                z[g] += p;
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[g][i] = fmaf(p, vf[i], acc[g][i]);
            }
        }
#pragma unroll
        for (int j = 0; j < kLoads; ++j) wc[j] = wn[j];
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
        for (int o = 16; o < 64; o <<= 1) {
            z[g] += __shfl_xor(z[g], o);
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[g][i] += __shfl_xor(acc[g][i], o);
        }
        if (r == 0) {
#pragma unroll
            for (int i = 0; i < 8; ++i) red_s[wave][g][cl * 8 + i] = acc[g][i];
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
        const size_t hq = size_t(b) * Hq + size_t(h) * G + g;
        const float res = o / zsum;
        if (a.out_dtype == 0) reinterpret_cast<float*>(a.out)[hq * kD + d] = res;
        else reinterpret_cast<_Float16*>(a.out)[hq * kD + d] = (_Float16)res;
    }
}

hipError_t launch_fp16(const akv_shape& s, const uint16_t* k, const uint16_t* v, const int32_t* lens, const uint16_t* q,
                       void* out, float scale, int out_dtype, int max_len, void* ws, hipStream_t st)
{
    F16Args a;
    a.s = s; a.k = k; a.v = v; a.q = q; a.lens = lens; a.out = out;
    a.c = (float)((double)scale * 1.4426950408889634);
    a.out_dtype = out_dtype;
    a.nsplit = f_splits(s.Ncap);
    a.max_len = max_len;
    const size_t bhq = size_t(s.B) * s.Hq;
    char* p = reinterpret_cast<char*>(ws);
    a.partO = reinterpret_cast<float*>(p);
    p += align256(bhq * a.nsplit * kD * sizeof(float));
    a.partM = reinterpret_cast<float*>(p);
    p += align256(bhq * a.nsplit * sizeof(float));
    a.partZ = reinterpret_cast<float*>(p);
    p += align256(bhq * a.nsplit * sizeof(float));
    float* logits = reinterpret_cast<float*>(p);
    const int G = s.Hq / s.Hkv;
    // One workgroup per head only for short sequences on a full chip (timed on 256 heads: 31.6 against 40.5 us at 1024
    // tokens, even at 2048, 99 against 86.5 us at 4096): beyond that the many small workgroups of the chunk kernel
    // stream faster (6.2 TB/s), and the yardstick is the faster of the two.
    if (G <= 2 && s.B * s.Hkv >= 192 && max_len < 2048) {
        const dim3 hgrid(xcd_grid(size_t(s.B) * s.Hkv));
        if (G == 1) hipLaunchKernelGGL((fp16_head_kernel<1, 1024>), hgrid, dim3(1024), 0, st, a, logits);
        else hipLaunchKernelGGL((fp16_head_kernel<2, 1024>), hgrid, dim3(1024), 0, st, a, logits);
        return hipGetLastError();
    }
    const dim3 grid(f_splits(max_len), s.Hkv, s.B), block(64 * kFWaves);
    switch (G) {
        case 1: hipLaunchKernelGGL(fp16_kernel<1>, grid, block, 0, st, a); break;
        case 2: hipLaunchKernelGGL(fp16_kernel<2>, grid, block, 0, st, a); break;
        case 4: hipLaunchKernelGGL(fp16_kernel<4>, grid, block, 0, st, a); break;
        case 8: hipLaunchKernelGGL(fp16_kernel<8>, grid, block, 0, st, a); break;
        default: return hipErrorInvalidValue;
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(fp16_combine_kernel, dim3(s.Hq, s.B), dim3(kD), 0, st, a);
    return hipGetLastError();
}

}  // namespace akv
