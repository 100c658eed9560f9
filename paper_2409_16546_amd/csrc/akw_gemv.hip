// Precision-aligned weight GEMV (declared in include/akw.h): y = x W with the rows of W read at the precision
// Rule 1 assigns them from x and rowmax.  "Precision Alignment in Uncertainty Calculation" (A W = A (W_quant +- dW)),
// "A Framework for Aligning Precision" (Rule 1; an addend's bit width is its weight's), "Dynamic Quantization"
// (first 8 / first 12 / all 16 bits, the rest counts as 100...).
//
// One kernel.  A workgroup (8 waves) owns a strip of 128 columns x 512 rows; a wave owns 64 of those rows, as
// eight groups of 8 rows; lane -> row lane/8 of the group and the 16-column slice lane%8, so one 16-byte load per
// lane fetches the 128 contiguous HI bytes of each of 8 rows (the MID and LO bytes: 8 bytes per lane; a row whose
// level does not need a plane is asked for out of range and fetches nothing).  All of a wave's loads are in flight
// at once: the HI bytes go first, before anything is known about the levels.  Every workgroup derives the largest
// addend exponent of each activation row from x and rowmax itself (K products, from L2) -- cheaper than a launch
// of its own in front of a kernel that runs for a few microseconds.  The sums over the 8 row lanes meet by lane
// exchange, the waves' sums in LDS, the slabs' sums (K/512 of them) in the workspace: the workgroup that draws
// the last ticket of a strip adds them in slab order, so the result does not depend on timing.
#include <cstdarg>

#include "../../include/akw.h"
#include "akv_common.h"

namespace akv {

constexpr int kWWaves = 8;                   // waves per workgroup
constexpr int kWThreads = 64 * kWWaves;
constexpr int kWCols = 128;                  // columns per workgroup: 16 per lane, 8 lanes per row
constexpr int kWGroups = 8;                  // groups of 8 rows per wave
constexpr int kWSlab = kWWaves * kWGroups * 8;   // rows per workgroup: 512
static_assert(AKW_MAX_B * kWCols <= kWThreads && kWSlab == kWThreads, "a thread per (activation row, column) and per slab row");

struct GemvArgs {
    int K, N, nslab;
    const uint8_t *hi, *mid, *lo;
    const uint16_t *rowmax, *x;
    float *y, *part;      // part: [nslab][B][N]
    int32_t* count;       // [column strips]
    int guard_bits, force_level;
    uint8_t* lvl_out;
};

template <int B>
__global__ __launch_bounds__(kWThreads, 4) void gemv_kernel(GemvArgs a)   // two workgroups per compute unit at least
{
    __shared__ int emax_s[B][kWWaves];
    __shared__ int lvl_s[kWSlab];
    __shared__ float xs[B][kWSlab];
    __shared__ float red_s[kWWaves][B][kWCols];
    __shared__ int last_s;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane >> 3, cl = lane & 7;
    const int strip = blockIdx.x, slab_i = blockIdx.y;
    const int K = a.K, N = a.N;
    const int col = strip * kWCols + cl * 16, k0 = slab_i * kWSlab;
    const bool lane_ok = col < N;                                   // N % 16 == 0: a lane is inside or outside as a whole

    const __amdgpu_buffer_rsrc_t rs_hi = make_rsrc(a.hi, uint32_t(K) * uint32_t(N));
    const __amdgpu_buffer_rsrc_t rs_mid = make_rsrc(a.mid, uint32_t(K) * uint32_t(N / 2));
    const __amdgpu_buffer_rsrc_t rs_lo = make_rsrc(a.lo, uint32_t(K) * uint32_t(N / 2));
    auto local_row = [&](int g) { return (wave * kWGroups + g) * 8 + r; };   // row of the slab this lane reads in group g

    // ---- the wave's HI bytes: in flight before anything is known about the levels (asked for first: the sooner the
    // stream of weights starts, the sooner it ends -- putting the few loads of the exponents in front of them
    // measured slower)
    u32x4_t H[kWGroups];
#pragma unroll
    for (int g = 0; g < kWGroups; ++g) {
        const int k = k0 + local_row(g);
        H[g] = buf_load_b128(rs_hi, lane_ok && k < K ? uint32_t(k) * uint32_t(N) + uint32_t(col) : kSkip);
    }

    // ---- Rule 1: largest addend exponent of every activation row, over all K input features (8 per thread and round)
    int emax[B];
#pragma unroll
    for (int b = 0; b < B; ++b) emax[b] = -1;
    const int nvec = K / 8;
    for (int v = tid; v < nvec; v += kWThreads) {
        const uint4 rm = reinterpret_cast<const uint4*>(a.rowmax)[v];
        const uint32_t rw[4] = {rm.x, rm.y, rm.z, rm.w};
#pragma unroll
        for (int b = 0; b < B; ++b) {
            const uint4 xv = reinterpret_cast<const uint4*>(a.x)[size_t(b) * nvec + v];
            const uint32_t xw[4] = {xv.x, xv.y, xv.z, xv.w};
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const uint32_t r16 = (rw[i >> 1] >> (16 * (i & 1))) & 0xFFFFu;
                const uint32_t x16 = (xw[i >> 1] >> (16 * (i & 1))) & 0xFFFFu;
                const float P = half_bits_to_float(x16) * half_bits_to_float(r16 < 0x0400u ? 0x0400u : r16);   // exact
                const int e = float_exp_field(P);
                emax[b] = (P != 0.0f && e > emax[b]) ? e : emax[b];
            }
        }
    }
#pragma unroll
    for (int b = 0; b < B; ++b) {
        const int m = (int)wave_max((float)emax[b]);                // small integers: exact as floats
        if (lane == 0) emax_s[b][wave] = m;
    }
    __syncthreads();
    {                                                               // thread -> row k0 + tid of the slab: level and activations
        const int k = k0 + tid;
        int level = 0;
#pragma unroll
        for (int b = 0; b < B; ++b) {
            int em = -1;
#pragma unroll
            for (int w = 0; w < kWWaves; ++w) em = emax_s[b][w] > em ? emax_s[b][w] : em;
            float xf = 0.0f;
            if (k < K) {
                const uint32_t x16 = a.x[size_t(b) * K + k], r16 = a.rowmax[k];
                xf = half_bits_to_float(x16);
                const float P = xf * half_bits_to_float(r16 < 0x0400u ? 0x0400u : r16);
                if (P != 0.0f) {
                    const int l = level_for_mantissa_bits(10 + a.guard_bits - (em - float_exp_field(P)));
                    level = l > level ? l : level;
                }
            }
            xs[b][tid] = xf;                                        // rows at or past K: 0
        }
        if (a.force_level >= 0) level = a.force_level;
        lvl_s[tid] = level;
        if (a.lvl_out && strip == 0 && k < K) a.lvl_out[k] = (uint8_t)level;
    }
    __syncthreads();

    // ---- the planes the levels ask for, then the multiply-adds
    u32x2_t M[kWGroups], L[kWGroups];
    int lv[kWGroups];
#pragma unroll
    for (int g = 0; g < kWGroups; ++g) {
        const int lr = local_row(g), k = k0 + lr;
        lv[g] = lvl_s[lr];
        const uint32_t off = uint32_t(k) * uint32_t(N / 2) + uint32_t(col / 2);
        const bool in = lane_ok && k < K;
        M[g] = buf_load_b64(rs_mid, in && lv[g] >= 1 ? off : kSkip);
        L[g] = buf_load_b64(rs_lo, in && lv[g] >= 2 ? off : kSkip);
    }
    float acc[B][16];
#pragma unroll
    for (int b = 0; b < B; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[b][i] = 0.0f;
#pragma unroll
    for (int g = 0; g < kWGroups; ++g) {
        const uint32_t fill = fill_for_level(lv[g]);
        uint32_t pa[4], pb[4];
        assemble8_fill(H[g].x, H[g].y, M[g].x, L[g].x, fill, pa);   // columns 0..7 of the lane
        assemble8_fill(H[g].z, H[g].w, M[g].y, L[g].y, fill, pb);   // columns 8..15
        const float v[16] = {lo_half(pa[0]), lo_half(pa[1]), hi_half(pa[0]), hi_half(pa[1]),
                             lo_half(pa[2]), lo_half(pa[3]), hi_half(pa[2]), hi_half(pa[3]),
                             lo_half(pb[0]), lo_half(pb[1]), hi_half(pb[0]), hi_half(pb[1]),
                             lo_half(pb[2]), lo_half(pb[3]), hi_half(pb[2]), hi_half(pb[3])};
        const int lr = local_row(g);
#pragma unroll
        for (int b = 0; b < B; ++b) {
            const float xf = xs[b][lr];
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[b][i] = fmaf(xf, v[i], acc[b][i]);
        }
    }

    // ---- sums: over the 8 row lanes by lane exchange, over the waves in LDS, over the slabs in the workspace
#pragma unroll
    for (int b = 0; b < B; ++b)
        for (int o = 8; o < 64; o <<= 1) {
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[b][i] += __shfl_xor(acc[b][i], o);
        }
    if (r == 0) {
#pragma unroll
        for (int b = 0; b < B; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) red_s[wave][b][cl * 16 + i] = acc[b][i];
    }
    __syncthreads();
    const int nslab = a.nslab;
    const int c_out = strip * kWCols + (tid % kWCols), b_out = tid / kWCols;   // thread -> one (activation row, column)
    const bool mine = tid < B * kWCols && c_out < N;
    if (mine) {
        float sum = 0.0f;
#pragma unroll
        for (int w = 0; w < kWWaves; ++w) sum += red_s[w][b_out][tid % kWCols];
        if (nslab == 1) a.y[size_t(b_out) * N + c_out] = sum;
        else store_agent(&a.part[(size_t(slab_i) * B + b_out) * N + c_out], sum);
    }
    if (nslab == 1) return;

    // ---- the workgroup that finishes last for this strip adds the slabs, in slab order
    stores_done();
    __syncthreads();
    if (tid == 0) last_s = take_ticket(&a.count[strip]) == nslab - 1;
    __syncthreads();
    if (!last_s) return;
    if (mine) {
        float sum = 0.0f;
        for (int s0 = 0; s0 < nslab; s0 += 8) {   // eight slabs' words in flight; the additions stay in slab order
            float p[8];
#pragma unroll
            for (int i = 0; i < 8; ++i)
                p[i] = s0 + i < nslab ? load_agent(&a.part[(size_t(s0 + i) * B + b_out) * N + c_out]) : 0.0f;
#pragma unroll
            for (int i = 0; i < 8; ++i) sum += p[i];
        }
        a.y[size_t(b_out) * N + c_out] = sum;
    }
    if (tid == 0) store_agent(&a.count[strip], 0);   // ready for the next call
}

// W [K][N] fp16 -> planes and rowmax: one workgroup per row, a thread packs 16 columns at a time
__global__ __launch_bounds__(256) void pack_kernel(int K, int N, const uint16_t* __restrict__ W, uint8_t* hi, uint8_t* mid,
                                                   uint8_t* lo, uint16_t* rowmax)
{
    __shared__ uint32_t mx_s[4];
    const int k = blockIdx.x, tid = threadIdx.x;
    uint32_t mx = 0;
    for (int c = tid * 16; c < N; c += 256 * 16) {
        const uint4 a = *reinterpret_cast<const uint4*>(W + size_t(k) * N + c);
        const uint4 b = *reinterpret_cast<const uint4*>(W + size_t(k) * N + c + 8);
        const uint32_t w[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};   // w[i] = columns 2i (low half), 2i+1 (high half)
        uint32_t h[4] = {0, 0, 0, 0}, m[2] = {0, 0}, l[2] = {0, 0};
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t e = w[i] & 0xFFFFu, o = w[i] >> 16;
            h[i >> 1] |= ((e >> 8) | ((o >> 8) << 8)) << (16 * (i & 1));
            m[i >> 2] |= (((e >> 4) & 15u) | (((o >> 4) & 15u) << 4)) << (8 * (i & 3));
            l[i >> 2] |= ((e & 15u) | ((o & 15u) << 4)) << (8 * (i & 3));
            const uint32_t me = e & 0x7FFFu, mo = o & 0x7FFFu;
            mx = me > mx ? me : mx;
            mx = mo > mx ? mo : mx;
        }
        *reinterpret_cast<uint4*>(hi + size_t(k) * N + c) = make_uint4(h[0], h[1], h[2], h[3]);
        *reinterpret_cast<uint2*>(mid + size_t(k) * (N / 2) + c / 2) = make_uint2(m[0], m[1]);
        *reinterpret_cast<uint2*>(lo + size_t(k) * (N / 2) + c / 2) = make_uint2(l[0], l[1]);
    }
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t other = (uint32_t)__shfl_xor((int)mx, o);
        mx = other > mx ? other : mx;
    }
    if ((tid & 63) == 0) mx_s[tid >> 6] = mx;
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < 4; ++w) mx = mx_s[w] > mx ? mx_s[w] : mx;
        rowmax[k] = (uint16_t)mx;
    }
}

__global__ __launch_bounds__(256) void unpack_kernel(int K, int N, const uint8_t* __restrict__ hi, const uint8_t* __restrict__ mid,
                                                     const uint8_t* __restrict__ lo, uint16_t* W)
{
    const int k = blockIdx.x;
    for (int c = threadIdx.x * 2; c < N; c += 512) {
        const uint32_t m = mid[size_t(k) * (N / 2) + c / 2], l = lo[size_t(k) * (N / 2) + c / 2];
        const uint32_t h0 = hi[size_t(k) * N + c], h1 = hi[size_t(k) * N + c + 1];
        const uint32_t e = (h0 << 8) | ((m & 15u) << 4) | (l & 15u), o = (h1 << 8) | ((m >> 4) << 4) | (l >> 4);
        *reinterpret_cast<uint32_t*>(W + size_t(k) * N + c) = e | (o << 16);
    }
}

}  // namespace akv

namespace {

bool wshape_ok(int K, int N)
{
    return K >= 8 && K % 8 == 0 && K <= (1 << 20) && N >= 16 && N % 16 == 0 && (long long)K * N < (1LL << 31);
}
size_t align256(size_t x) { return (x + 255) / 256 * 256; }
bool aligned16(const void* p) { return reinterpret_cast<uintptr_t>(p) % 16 == 0; }
size_t part_bytes(int K, int N)
{
    return align256(size_t((K + akv::kWSlab - 1) / akv::kWSlab) * AKW_MAX_B * size_t(N) * sizeof(float));
}
size_t count_bytes(int N) { return align256(size_t((N + akv::kWCols - 1) / akv::kWCols) * sizeof(int32_t)); }

akv_status check_weights(const akw_weights* w)
{
    if (!w) return akv::fail_msg(AKV_EINVAL, "weights is NULL");
    if (!wshape_ok(w->K, w->N))
        return akv::fail_msg(AKV_EINVAL, "bad shape: K=%d N=%d (need K %% 8 == 0, K <= 2^20, N %% 16 == 0, K*N < 2^31)", w->K, w->N);
    if (!w->hi || !w->mid || !w->lo || !w->rowmax) return akv::fail_msg(AKV_EINVAL, "weights has a NULL plane / rowmax pointer");
    if (!aligned16(w->hi) || !aligned16(w->mid) || !aligned16(w->lo) || !aligned16(w->rowmax))
        return akv::fail_msg(AKV_EINVAL, "the planes and rowmax must be 16-byte aligned");
    return AKV_OK;
}

}  // namespace

extern "C" {

akv_status akw_layout_sizes(int32_t K, int32_t N, akw_sizes* out)
{
    if (!out) return akv::fail_msg(AKV_EINVAL, "NULL argument");
    if (!wshape_ok(K, N)) return akv::fail_msg(AKV_EINVAL, "bad shape: K=%d N=%d (need K %% 8 == 0, K <= 2^20, N %% 16 == 0, K*N < 2^31)", K, N);
    out->hi = size_t(K) * N;
    out->mid = out->lo = size_t(K) * (N / 2);
    out->rowmax = size_t(K) * sizeof(uint16_t);
    out->workspace = part_bytes(K, N) + count_bytes(N);
    return AKV_OK;
}

akv_status akw_workspace_init(int32_t K, int32_t N, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!wshape_ok(K, N)) return akv::fail_msg(AKV_EINVAL, "bad shape: K=%d N=%d", K, N);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) || workspace_bytes < part_bytes(K, N) + count_bytes(N))
        return akv::fail_msg(AKV_EWORKSPACE, "workspace NULL, misaligned or smaller than %zu bytes", part_bytes(K, N) + count_bytes(N));
    if (hipError_t e = akv::launch_zero(static_cast<char*>(workspace) + part_bytes(K, N), count_bytes(N), static_cast<hipStream_t>(stream)))
        return akv::fail_msg(AKV_EHIP, "workspace init launch: %s", hipGetErrorString(e));
    return AKV_OK;
}

akv_status akw_pack(const akw_weights* w, const uint16_t* W, void* stream)
{
    if (akv_status st = check_weights(w)) return st;
    if (!W || !aligned16(W)) return akv::fail_msg(AKV_EINVAL, "W is NULL or not 16-byte aligned");
    hipLaunchKernelGGL(akv::pack_kernel, dim3(w->K), dim3(256), 0, static_cast<hipStream_t>(stream), w->K, w->N, W, w->hi, w->mid,
                       w->lo, w->rowmax);
    if (hipError_t e = hipGetLastError()) return akv::fail_msg(AKV_EHIP, "pack launch: %s", hipGetErrorString(e));
    return AKV_OK;
}

akv_status akw_unpack(const akw_weights* w, uint16_t* W_out, void* stream)
{
    if (akv_status st = check_weights(w)) return st;
    if (!W_out || !aligned16(W_out)) return akv::fail_msg(AKV_EINVAL, "W_out is NULL or not 16-byte aligned");
    hipLaunchKernelGGL(akv::unpack_kernel, dim3(w->K), dim3(256), 0, static_cast<hipStream_t>(stream), w->K, w->N, w->hi, w->mid,
                       w->lo, W_out);
    if (hipError_t e = hipGetLastError()) return akv::fail_msg(AKV_EHIP, "unpack launch: %s", hipGetErrorString(e));
    return AKV_OK;
}

akv_status akw_gemv(const akw_weights* w, const uint16_t* x, int32_t B, float* y, const akw_params* params, void* workspace,
                    size_t workspace_bytes, void* stream)
{
    if (akv_status st = check_weights(w)) return st;
    if (!x || !y) return akv::fail_msg(AKV_EINVAL, "x / y is NULL");
    if (!aligned16(x) || !aligned16(y)) return akv::fail_msg(AKV_EINVAL, "x and y must be 16-byte aligned");
    if (B < 1 || B > AKW_MAX_B) return akv::fail_msg(AKV_EINVAL, "B = %d out of range 1..%d", B, AKW_MAX_B);
    akw_params p = {0, -1, nullptr};
    if (params) p = *params;
    if (p.guard_bits < 0 || p.guard_bits > 12) return akv::fail_msg(AKV_EINVAL, "guard_bits = %d out of range 0..12", p.guard_bits);
    if (p.force_level < -1 || p.force_level > 2) return akv::fail_msg(AKV_EINVAL, "force_level = %d out of range -1..2", p.force_level);
    const size_t need = part_bytes(w->K, w->N) + count_bytes(w->N);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) || workspace_bytes < need)
        return akv::fail_msg(AKV_EWORKSPACE, "workspace NULL, misaligned or smaller than %zu bytes", need);
    akv::GemvArgs a;
    a.K = w->K; a.N = w->N;
    a.nslab = (w->K + akv::kWSlab - 1) / akv::kWSlab;
    a.hi = w->hi; a.mid = w->mid; a.lo = w->lo; a.rowmax = w->rowmax; a.x = x; a.y = y;
    a.part = static_cast<float*>(workspace);
    a.count = reinterpret_cast<int32_t*>(static_cast<char*>(workspace) + part_bytes(w->K, w->N));
    a.guard_bits = p.guard_bits; a.force_level = p.force_level; a.lvl_out = p.lvl_out;
    const dim3 grid((w->N + akv::kWCols - 1) / akv::kWCols, a.nslab), block(akv::kWThreads);
    hipStream_t st = static_cast<hipStream_t>(stream);
    switch (B) {
        case 1: hipLaunchKernelGGL(akv::gemv_kernel<1>, grid, block, 0, st, a); break;
        case 2: hipLaunchKernelGGL(akv::gemv_kernel<2>, grid, block, 0, st, a); break;
        case 3: hipLaunchKernelGGL(akv::gemv_kernel<3>, grid, block, 0, st, a); break;
        default: hipLaunchKernelGGL(akv::gemv_kernel<4>, grid, block, 0, st, a); break;
    }
    if (hipError_t e = hipGetLastError()) return akv::fail_msg(AKV_EHIP, "gemv launch: %s", hipGetErrorString(e));
    return AKV_OK;
}

}  // extern "C"
