// Append tokens into the split-plane cache and its inverse.
// "Dynamic Quantization": the cache keeps all 16 bits of every element, the first 8 / next 4 / last 4
// bits in separately contiguous planes; "Quantization of K-Cache": K_colmax is kept while storing.
#include "akv_common.h"

namespace akv {

// One workgroup per (sequence, KV head), 128 threads: thread d owns K channel d (so it is the only writer
// of that column's nibble bytes and of colmax[d]); threads 0..63 own the V nibble byte of channels 2d, 2d+1.
// flags[AKV_NFLAGS + b] counts the workgroups of sequence b that are done (zero between calls).
__global__ __launch_bounds__(128) void append_kernel(akv_cache c, const uint16_t* __restrict__ k_new,
                                                     const uint16_t* __restrict__ v_new,
                                                     const int32_t* __restrict__ n_new, int n)
{
    const int h = blockIdx.x, b = blockIdx.y, d = threadIdx.x;
    const int Hkv = c.shape.Hkv, Ncap = c.shape.Ncap;
    const int len = c.lens[b];
    int cnt = n_new ? n_new[b] : n;
    cnt = cnt < 0 ? 0 : (cnt > n ? n : cnt);
    const bool fits = len + cnt <= Ncap;   // else the sequence is left unchanged and the refusal is counted
    const size_t bh = size_t(b) * Hkv + h;
    // The ticket is drawn as soon as this workgroup has read the length (the test keeps the atomic behind that read):
    // its round trip then runs beside the loads and stores below instead of after them.  Whoever draws the last one
    // moves the length at its end -- every head of the sequence has read the old one by then, and nothing in this
    // kernel reads the planes.
    int ticket = -1;
    if (d == 0 && len >= 0) ticket = atomicAdd(&c.flags[AKV_NFLAGS + b], 1);
    if (fits) {
    const uint16_t* kn = k_new + bh * n * kD;
    const uint16_t* vn = v_new + bh * n * kD;
    uint32_t cm = c.colmax[bh * kD + d];
    for (int i = 0; i < cnt; ++i) {
        const uint32_t mag = store_token(c.k_hi, c.k_mid, c.k_lo, c.v_hi, c.v_mid, c.v_lo, bh, Ncap, len + i, d,
                                         kn + size_t(i) * kD, vn + size_t(i) * kD);
        cm = mag > cm ? mag : cm;
    }
    c.colmax[bh * kD + d] = (uint16_t)cm;
    }
    if (d == 0 && ticket == Hkv - 1) {
        c.flags[AKV_NFLAGS + b] = 0;
        if (fits) c.lens[b] = len + cnt;
        else atomicAdd(&c.flags[AKV_FLAG_OVERFLOW], 1);
    }
}

// Bulk append (prefill): one workgroup of 256 threads per (sequence, KV head, 256-token K block touched).
// V rows need no transposition: a thread turns 16 channels of a row (32 bytes in) into 16 + 8 + 8 bytes of the three
// planes.  A K block that the new tokens cover completely goes through an LDS tile [256 tokens][128 channels] and
// leaves as 16-byte pieces of the channel-major runs; a block they cover only partly (the first one after a
// sequence that does not end on a block boundary, the last one) is stored token by token, thread d being the only
// writer of column d.  K_colmax: a 16-bit maximum through compare-and-swap on the enclosing word.
constexpr int kTilePad = kD + 2;   // halves per token row of the LDS tile: rows 65 words apart, columns conflict-free

__device__ __forceinline__ void colmax_update(uint16_t* colmax, size_t idx, uint32_t mag)
{
    uint32_t* word = reinterpret_cast<uint32_t*>(colmax + (idx & ~size_t(1)));
    const int sh = (idx & 1) ? 16 : 0;
    uint32_t old = *word;
    while (((old >> sh) & 0xFFFFu) < mag) {
        const uint32_t want = (old & ~(0xFFFFu << sh)) | (mag << sh);
        const uint32_t seen = atomicCAS(word, old, want);
        if (seen == old) break;
        old = seen;
    }
}

__global__ __launch_bounds__(256) void append_block_kernel(akv_cache c, const uint16_t* __restrict__ k_new,
                                                           const uint16_t* __restrict__ v_new,
                                                           const int32_t* __restrict__ n_new, int n)
{
    __shared__ uint16_t tile[kTB][kTilePad];
    __shared__ int last_s;
    const int h = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
    const int Hkv = c.shape.Hkv, Ncap = c.shape.Ncap, NB = Ncap / kTB;
    const int len = c.lens[b];
    int cnt = n_new ? n_new[b] : n;
    cnt = cnt < 0 ? 0 : (cnt > n ? n : cnt);
    const bool fits = len + cnt <= Ncap;   // else the sequence is left unchanged and the refusal is counted
    const int first_blk = len / kTB;
    const int touched = cnt > 0 ? (len % kTB + cnt + kTB - 1) / kTB : 0;   // K blocks the new tokens fall into
    const int nwg = fits ? touched : (cnt > 0 ? 1 : 0);                    // workgroups per head that have work (or count the refusal)
    if ((int)blockIdx.x >= nwg) return;
    const size_t bh = size_t(b) * Hkv + h;
    if (fits) {
        const int blk = first_blk + blockIdx.x;
        const int t_lo = max(len, blk * kTB), t_hi = min(len + cnt, (blk + 1) * kTB);   // tokens of this block: [t_lo, t_hi)
        const uint16_t* kn = k_new + bh * n * kD;   // row i of the input is token len + i
        const uint16_t* vn = v_new + bh * n * kD;
        // ---- V: thread -> (row, 16 channels), 16 rows per pass ----
        for (int t = t_lo + (tid >> 3); t < t_hi; t += 32) {
            const int cl = tid & 7;
            const uint4* src = reinterpret_cast<const uint4*>(vn + size_t(t - len) * kD + cl * 16);
            const uint4 x0 = src[0], x1 = src[1];
            const uint32_t w[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};   // word i: channels 2i (low half), 2i+1
            uint32_t hi[4] = {0, 0, 0, 0}, mid[2] = {0, 0}, lo[2] = {0, 0};
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const uint32_t e0 = w[i] & 0xFFFFu, e1 = w[i] >> 16;
                hi[i / 2] |= ((e0 >> 8) | ((e1 >> 8) << 8)) << (16 * (i & 1));
                mid[i / 4] |= (((e0 >> 4) & 15u) | (((e1 >> 4) & 15u) << 4)) << (8 * (i & 3));
                lo[i / 4] |= ((e0 & 15u) | ((e1 & 15u) << 4)) << (8 * (i & 3));
            }
            const size_t row = bh * Ncap + t;
            *reinterpret_cast<uint4*>(c.v_hi + row * kD + cl * 16) = make_uint4(hi[0], hi[1], hi[2], hi[3]);
            *reinterpret_cast<uint2*>(c.v_mid + row * (kD / 2) + cl * 8) = make_uint2(mid[0], mid[1]);
            *reinterpret_cast<uint2*>(c.v_lo + row * (kD / 2) + cl * 8) = make_uint2(lo[0], lo[1]);
        }
        // ---- K ----
        if (t_hi - t_lo == kTB) {   // the whole block: through the LDS tile
            for (int idx = tid; idx < kTB * (kD / 8); idx += 256) {   // 16-byte pieces of the input rows
                const int j = idx / (kD / 8), p8 = idx % (kD / 8);
                const uint4 x = *reinterpret_cast<const uint4*>(kn + size_t(t_lo - len + j) * kD + p8 * 8);
                uint32_t* dst = reinterpret_cast<uint32_t*>(&tile[j][p8 * 8]);   // rows start at even halves: word aligned
                dst[0] = x.x; dst[1] = x.y; dst[2] = x.z; dst[3] = x.w;
            }
            __syncthreads();
            const size_t colbase = (bh * NB + blk) * kD;
            for (int idx = tid; idx < kD * (kTB / 16); idx += 256) {   // HI: (column d, 16 tokens) -> 16 bytes
                const int d = idx / (kTB / 16), j0 = (idx % (kTB / 16)) * 16;
                uint32_t o[4] = {0, 0, 0, 0};
#pragma unroll
                for (int i = 0; i < 16; ++i) o[i / 4] |= uint32_t(tile[j0 + i][d] >> 8) << (8 * (i & 3));
                *reinterpret_cast<uint4*>(c.k_hi + (colbase + d) * kTB + j0) = make_uint4(o[0], o[1], o[2], o[3]);
            }
            for (int idx = tid; idx < kD * (kTB / 32); idx += 256) {   // MID, LO: (column d, 32 tokens) -> 16 bytes each
                const int d = idx / (kTB / 32), j0 = (idx % (kTB / 32)) * 32;
                uint32_t m[4] = {0, 0, 0, 0}, l[4] = {0, 0, 0, 0};
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const uint32_t e0 = tile[j0 + 2 * i][d], e1 = tile[j0 + 2 * i + 1][d];
                    m[i / 4] |= (((e0 >> 4) & 15u) | (((e1 >> 4) & 15u) << 4)) << (8 * (i & 3));
                    l[i / 4] |= ((e0 & 15u) | ((e1 & 15u) << 4)) << (8 * (i & 3));
                }
                *reinterpret_cast<uint4*>(c.k_mid + (colbase + d) * (kTB / 2) + j0 / 2) = make_uint4(m[0], m[1], m[2], m[3]);
                *reinterpret_cast<uint4*>(c.k_lo + (colbase + d) * (kTB / 2) + j0 / 2) = make_uint4(l[0], l[1], l[2], l[3]);
            }
            if (tid < kD) {
                uint32_t mag = 0;
                for (int j = 0; j < kTB; ++j) mag = max(mag, uint32_t(tile[j][tid]) & 0x7FFFu);
                colmax_update(c.colmax, bh * kD + tid, mag);
            }
        } else if (tid < kD) {      // part of a block: token by token, thread d owns column d
            uint32_t mag = 0;
            for (int t = t_lo; t < t_hi; ++t) {
                const uint32_t kx = kn[size_t(t - len) * kD + tid];
                const int j = t % kTB;
                const size_t col = (bh * NB + blk) * kD + tid;
                c.k_hi[col * kTB + j] = (uint8_t)(kx >> 8);
                const size_t nib = col * (kTB / 2) + j / 2;
                const uint32_t om = c.k_mid[nib], ol = c.k_lo[nib];
                if (j & 1) {
                    c.k_mid[nib] = (uint8_t)((om & 0x0F) | (((kx >> 4) & 15u) << 4));
                    c.k_lo[nib] = (uint8_t)((ol & 0x0F) | ((kx & 15u) << 4));
                } else {
                    c.k_mid[nib] = (uint8_t)((om & 0xF0) | ((kx >> 4) & 15u));
                    c.k_lo[nib] = (uint8_t)((ol & 0xF0) | (kx & 15u));
                }
                mag = max(mag, kx & 0x7FFFu);
            }
            colmax_update(c.colmax, bh * kD + tid, mag);
        }
    }
    // The workgroup of the sequence that arrives last (every one has read lens[b] by then) moves the length.
    __syncthreads();
    if (tid == 0) last_s = atomicAdd(&c.flags[AKV_NFLAGS + b], 1) == nwg * Hkv - 1;
    __syncthreads();
    if (last_s && tid == 0) {
        c.flags[AKV_NFLAGS + b] = 0;
        if (fits) c.lens[b] = len + cnt;
        else atomicAdd(&c.flags[AKV_FLAG_OVERFLOW], 1);
    }
}

hipError_t launch_append(const akv_cache& c, const uint16_t* k_new, const uint16_t* v_new, const int32_t* n_new, int n,
                         hipStream_t st)
{
    if (n == 0) return hipSuccess;
    if (n < 32) {   // a few tokens: one workgroup per (sequence, KV head) walks them
        hipLaunchKernelGGL(append_kernel, dim3(c.shape.Hkv, c.shape.B), dim3(128), 0, st, c, k_new, v_new, n_new, n);
    } else {        // prefill: a workgroup per K block; n tokens touch at most n / 256 + 2 blocks
        hipLaunchKernelGGL(append_block_kernel, dim3(n / kTB + 2, c.shape.Hkv, c.shape.B), dim3(256), 0, st, c, k_new, v_new, n_new, n);
    }
    return hipGetLastError();
}

// planes -> fp16 [B][Hkv][Ncap][D]; one thread per (token, channel pair)
__global__ __launch_bounds__(256) void unpack_kernel(akv_cache c, uint16_t* __restrict__ k_out,
                                                     uint16_t* __restrict__ v_out)
{
    const int Hkv = c.shape.Hkv, Ncap = c.shape.Ncap, NB = Ncap / kTB;
    const size_t idx = size_t(blockIdx.x) * 256 + threadIdx.x;          // over B*Hkv*Ncap*(D/2)
    const size_t total = size_t(c.shape.B) * Hkv * Ncap * (kD / 2);
    if (idx >= total) return;
    const int dp = int(idx % (kD / 2));
    const size_t row = idx / (kD / 2);                                   // (b*Hkv + h)*Ncap + t
    const int t = int(row % Ncap);
    const size_t bh = row / Ncap;
    if (v_out) {
        const uint32_t h0 = c.v_hi[row * kD + 2 * dp], h1 = c.v_hi[row * kD + 2 * dp + 1];
        const uint32_t m = c.v_mid[row * (kD / 2) + dp], l = c.v_lo[row * (kD / 2) + dp];
        v_out[row * kD + 2 * dp] = (uint16_t)((h0 << 8) | ((m & 15u) << 4) | (l & 15u));
        v_out[row * kD + 2 * dp + 1] = (uint16_t)((h1 << 8) | ((m >> 4) << 4) | (l >> 4));
    }
    if (k_out) {
        const int blk = t / kTB, j = t % kTB;
        for (int u = 0; u < 2; ++u) {
            const int d = 2 * dp + u;
            const size_t col = (bh * NB + blk) * kD + d;
            const uint32_t hi = c.k_hi[col * kTB + j];
            const uint32_t m = c.k_mid[col * (kTB / 2) + j / 2], l = c.k_lo[col * (kTB / 2) + j / 2];
            const uint32_t mn = (j & 1) ? (m >> 4) : (m & 15u), ln = (j & 1) ? (l >> 4) : (l & 15u);
            k_out[row * kD + d] = (uint16_t)((hi << 8) | (mn << 4) | ln);
        }
    }
}

hipError_t launch_unpack(const akv_cache& c, uint16_t* k_out, uint16_t* v_out, hipStream_t st)
{
    const size_t total = size_t(c.shape.B) * c.shape.Hkv * c.shape.Ncap * (kD / 2);
    hipLaunchKernelGGL(unpack_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, c, k_out, v_out);
    return hipGetLastError();
}

// zero a buffer with 16-byte stores (a kernel rather than a memset node, so that a caller may capture it)
__global__ __launch_bounds__(256) void zero_kernel(uint4* __restrict__ p16, size_t n16, uint8_t* __restrict__ tail,
                                                   int ntail)
{
    const size_t stride = size_t(gridDim.x) * 256;
    for (size_t i = size_t(blockIdx.x) * 256 + threadIdx.x; i < n16; i += stride) p16[i] = make_uint4(0, 0, 0, 0);
    if (blockIdx.x == 0 && (int)threadIdx.x < ntail) tail[threadIdx.x] = 0;
}

hipError_t launch_zero(void* p, size_t bytes, hipStream_t st)
{
    if (bytes == 0) return hipSuccess;
    const size_t n16 = bytes / 16;   // buffers come from an allocator: 16-byte aligned
    size_t blocks = (n16 + 255) / 256;
    blocks = blocks < 1 ? 1 : (blocks > 8192 ? 8192 : blocks);
    hipLaunchKernelGGL(zero_kernel, dim3((unsigned)blocks), dim3(256), 0, st, reinterpret_cast<uint4*>(p), n16,
                       reinterpret_cast<uint8_t*>(p) + n16 * 16, int(bytes - n16 * 16));
    return hipGetLastError();
}

// Plain streaming read (16 bytes per lane with the non-temporal hint, four loads in flight per lane): the read ceiling of the
// device that the roofline fractions of the other kernels are put beside.
__global__ __launch_bounds__(256) void stream_read_kernel(const uint4* __restrict__ p, size_t n16, uint32_t* sink)
{
    auto ld = [](const uint4* q) {   // non-temporal, as the decode kernels read the bytes they stream
        const u32x4_t w = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(q));
        return make_uint4(w.x, w.y, w.z, w.w);
    };
    // 4-KB chunks (one per workgroup and step) in blocks of 1 MB that go to the XCDs in turn (workgroup L runs on XCD
    // L % 8): an XCD reads stretches, as in the decode kernels -- chunks dealt singly over the XCDs read 15 % slower
    constexpr size_t kCpb = 256;   // chunks per block
    const size_t nchunks = (n16 + 255) / 256, x = blockIdx.x % kXcds, per = gridDim.x / kXcds;
    auto at = [&](size_t n) { return (((n / kCpb) * kXcds + x) * kCpb + n % kCpb) * 256 + threadIdx.x; };   // vector of chunk n of this XCD
    const uint4 zero = make_uint4(0, 0, 0, 0);
    uint32_t acc = 0;
    for (size_t n = blockIdx.x / kXcds; (n / kCpb) * kXcds * kCpb < nchunks; n += 4 * per) {
        const size_t i0 = at(n), i1 = at(n + per), i2 = at(n + 2 * per), i3 = at(n + 3 * per);
        const uint4 a = i0 < n16 ? ld(p + i0) : zero, b = i1 < n16 ? ld(p + i1) : zero;
        const uint4 c = i2 < n16 ? ld(p + i2) : zero, d = i3 < n16 ? ld(p + i3) : zero;
        acc += a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
    }
    if (acc == 0x9E3779B9u) *sink = acc;   // keeps the loads alive; practically never taken
}

hipError_t launch_stream_read(const void* p, size_t bytes, uint32_t* sink, hipStream_t st)
{
    const size_t n16 = bytes / 16;
    if (n16 == 0) return hipSuccess;
    size_t blocks = (n16 + 1023) / 1024;
    blocks = blocks < 1 ? 1 : (blocks > 8192 ? 8192 : blocks);
    hipLaunchKernelGGL(stream_read_kernel, dim3(xcd_grid(blocks)), dim3(256), 0, st, reinterpret_cast<const uint4*>(p), n16, sink);
    return hipGetLastError();
}

}  // namespace akv
