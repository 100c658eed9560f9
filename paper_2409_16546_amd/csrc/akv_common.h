// Shared declarations of the AlignedKV HIP library (host launchers + device helpers).
// Rules and layout: include/akv.h.  Paper sections are cited where an operation is defined.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/akv.h"

namespace akv {

constexpr int kD = 128;            // head dimension ("Runtime of AlignedKV": sqrt(128))
constexpr int kTB = AKV_TB;        // tokens per K block
constexpr int kAMin = -64;         // floor of the score exponent
constexpr int kBuckets = 65;       // exponent buckets 0..64 of the approximate top-k
constexpr int kMaxG = 8;           // query heads per KV head supported

// K pass: one wave covers one 256-token block (4 consecutive tokens per lane).
constexpr int kKWaves = 4;                         // waves per workgroup
constexpr int kMidSlice = kTB * kKWaves;           // tokens per workgroup of the K kernel and of the slice kernel
constexpr int kHistStride = 66;                    // ints per slice histogram in the workspace (65 buckets)
// V pass: one workgroup covers kVChunk tokens; a wave reads 8 token rows per step.
constexpr int kVWaves = 4;
constexpr int kVChunk = 512;

// Offsets (bytes) into the decode workspace.
struct WsLayout {
    size_t logits;   // float [B][Hq][Ncap]
    size_t tilemax;  // float [B][Hq][Ncap / 256]: per-wave-tile maxima of the K pass
    size_t M;        // float [B][Hq]
    size_t hist;     // int32 [B][Hq][ceil(Ncap / 1024)][66]: per-slice histograms of score exponents (token-split path)
    size_t cand_sel; // int32 [B][Hq][ceil(Ncap / 1024)][64]: per-slice top-k candidates, token | bucket << 24 (token-split path)
    size_t cand_phat;// float, same shape: their weights
    size_t Ehat;     // int32 [B][Hkv][D]
    size_t partO;    // float [B][Hq][v_splits(Ncap)][D]
    size_t partZ;    // float [B][Hq][v_splits(Ncap)]
    size_t control;  // int32 [2][B][Hkv]: a spare word and the arrival counter of the V kernel per (sequence, KV head); zero between calls
    size_t control_bytes;
    size_t total;
};

inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }
inline __host__ __device__ int v_splits(int ntok) { return (ntok + kVChunk - 1) / kVChunk; }   // V-pass chunks covering ntok

// control_front: the control words come first, inside a reserved block of kCtlReserve bytes whose place does not
// depend on the shape (the layout of the library's own static scratch array, shared by calls of every shape)
constexpr size_t kCtlReserve = 64 * 1024;
inline WsLayout ws_layout(const akv_shape& s, bool control_front = false)
{
    WsLayout w;
    size_t off = control_front ? kCtlReserve : 0;
    const size_t bhq = size_t(s.B) * s.Hq;
    w.logits = off;  off = align256(off + bhq * s.Ncap * sizeof(float));
    w.tilemax = off; off = align256(off + bhq * (s.Ncap / kTB) * sizeof(float));
    w.M = off;       off = align256(off + bhq * sizeof(float));
    w.hist = off;    off = align256(off + bhq * ((s.Ncap + kMidSlice - 1) / kMidSlice) * kHistStride * sizeof(int32_t));
    w.cand_sel = off; off = align256(off + bhq * ((s.Ncap + kMidSlice - 1) / kMidSlice) * AKV_MAX_TOPK * sizeof(int32_t));
    w.cand_phat = off; off = align256(off + bhq * ((s.Ncap + kMidSlice - 1) / kMidSlice) * AKV_MAX_TOPK * sizeof(float));
    w.Ehat = off;    off = align256(off + size_t(s.B) * s.Hkv * kD * sizeof(int32_t));
    w.partO = off;   off = align256(off + bhq * v_splits(s.Ncap) * kD * sizeof(float));
    w.partZ = off;   off = align256(off + bhq * v_splits(s.Ncap) * sizeof(float));
    w.control_bytes = 2 * size_t(s.B) * s.Hkv * sizeof(int32_t);
    if (control_front) {
        w.control = 0;
    } else {
        w.control = off;
        off = align256(off + w.control_bytes);
    }
    w.total = off;
    return w;
}

// Everything a decode kernel needs, passed by value.
struct DecodeArgs {
    akv_shape s;
    const uint8_t *k_hi, *k_mid, *k_lo, *v_hi, *v_mid, *v_lo;
    const uint16_t* colmax;
    const int32_t* lens;
    const uint16_t* q;
    const uint16_t *k_new, *v_new;   // fused append of one token per sequence ([B][Hkv][D] each), or NULL
    int32_t* flags;                  // cache flags (append arrival counters, overflow count); used with k_new
    void* out;
    float c;             // (float)(scale * log2(e))
    int topk, guard_bits, force_level, out_dtype, max_len;
    float* logits;       // [B][Hq][Ncap]
    float* tilemax;
    float* M;
    int32_t* Ehat;
    float* partO;
    float* partZ;
    int vchunk;          // tokens per workgroup of the V kernel of the token-split path (a multiple of 64: whole batches of rows for every wave; at least kVChunk)
    int32_t* hist;       // per-slice histograms of the token-split path
    int32_t* cand_sel;   // per-slice candidates of the token-split path
    float* cand_phat;
    int32_t* kcount;     // [B][Hkv] spare control words (kept zero; the selection runs in a kernel of its own)
    int32_t* vcount;
    akv_debug dbg;       // device pointers or NULL
    akv_stats* stats;    // device counters the kernels add to, or NULL
};

// Store one token of one (sequence, KV head) at position t: thread d (0..127) owns K channel d and is the
// only writer of that column's nibble bytes; threads 0..63 own the V nibble byte of channels 2d, 2d+1.
// Returns |k| as bits (for K_colmax).  "Dynamic Quantization": all 16 bits are kept, in three planes.
#if defined(__HIPCC__)
// byte index (within k_mid / k_lo) of the nibble pair that holds token t of column d
__device__ __forceinline__ size_t k_nibble_index(size_t bh, int Ncap, int t, int d)
{
    return ((bh * (Ncap / kTB) + t / kTB) * kD + d) * (kTB / 2) + (t % kTB) / 2;
}
// old_m, old_l: the current bytes at k_nibble_index (read by the caller, possibly long before)
__device__ __forceinline__ uint32_t store_token_rmw(uint8_t* k_hi, uint8_t* k_mid, uint8_t* k_lo, uint8_t* v_hi,
                                                    uint8_t* v_mid, uint8_t* v_lo, size_t bh, int Ncap, int t, int d,
                                                    const uint16_t* krow, const uint16_t* vrow, uint32_t old_m,
                                                    uint32_t old_l)
{
    const int NB = Ncap / kTB, blk = t / kTB, j = t % kTB;
    const uint32_t kx = krow[d];
    const size_t col = (bh * NB + blk) * kD + d;
    k_hi[col * kTB + j] = (uint8_t)(kx >> 8);
    const size_t nib = k_nibble_index(bh, Ncap, t, d);
    if (j & 1) {
        k_mid[nib] = (uint8_t)((old_m & 0x0F) | (((kx >> 4) & 15u) << 4));
        k_lo[nib] = (uint8_t)((old_l & 0x0F) | ((kx & 15u) << 4));
    } else {
        k_mid[nib] = (uint8_t)((old_m & 0xF0) | ((kx >> 4) & 15u));
        k_lo[nib] = (uint8_t)((old_l & 0xF0) | (kx & 15u));
    }
    const size_t row = bh * Ncap + t;
    const uint32_t vx = vrow[d];
    v_hi[row * kD + d] = (uint8_t)(vx >> 8);
    if (d < kD / 2) {
        const uint32_t v0 = vrow[2 * d], v1 = vrow[2 * d + 1];
        v_mid[row * (kD / 2) + d] = (uint8_t)(((v0 >> 4) & 15u) | (((v1 >> 4) & 15u) << 4));
        v_lo[row * (kD / 2) + d] = (uint8_t)((v0 & 15u) | ((v1 & 15u) << 4));
    }
    return kx & 0x7FFFu;   // |k| as bits: integer order is magnitude order
}
__device__ __forceinline__ uint32_t store_token(uint8_t* k_hi, uint8_t* k_mid, uint8_t* k_lo, uint8_t* v_hi,
                                                uint8_t* v_mid, uint8_t* v_lo, size_t bh, int Ncap, int t, int d,
                                                const uint16_t* krow, const uint16_t* vrow)
{
    const size_t nib = k_nibble_index(bh, Ncap, t, d);
    return store_token_rmw(k_hi, k_mid, k_lo, v_hi, v_mid, v_lo, bh, Ncap, t, d, krow, vrow, k_mid[nib], k_lo[nib]);
}
#endif

// host side: the error record, the device's size, and the launchers (each defined next to its kernels)
akv_status fail_msg(akv_status st, const char* fmt, ...);   // records the text akv_last_error() returns
int compute_units();                                         // of the current device (256 on MI355X), looked up once
hipError_t launch_append(const akv_cache& c, const uint16_t* k_new, const uint16_t* v_new, const int32_t* n_new, int n,
                         hipStream_t st);
hipError_t launch_zero(void* p, size_t bytes, hipStream_t st);
hipError_t launch_stream_read(const void* p, size_t bytes, uint32_t* sink, hipStream_t st);
hipError_t launch_unpack(const akv_cache& c, uint16_t* k_out, uint16_t* v_out, hipStream_t st);
hipError_t launch_decode_split(const DecodeArgs& a, hipStream_t st, hipEvent_t k_done_event, hipEvent_t mid_event);   // four kernels; the events (may be null) are recorded after the first and in front of the last
hipError_t launch_decode_head(const DecodeArgs& a, hipStream_t st);                         // one kernel, a head per workgroup
int split_v_workgroups_per_cu(int G);   // resident workgroups of the token-split V kernel per compute unit (registers, LDS)
bool head_path_supported(const akv_shape& s);
bool head_logits_in_lds(const akv_shape& s, int max_len);   // the head kernel keeps the logits of this shape in LDS (none written to memory)
hipError_t launch_fp16(const akv_shape& s, const uint16_t* k, const uint16_t* v, const int32_t* lens, const uint16_t* q,
                       void* out, float scale, int out_dtype, int max_len, void* ws, hipStream_t st);
size_t fp16_workspace_bytes(const akv_shape& s);

// Workgroups of a launch are dealt to the eight XCDs in turn: workgroup L of a one-dimensional grid runs on XCD
// L % 8.  The streaming kernels give every XCD one contiguous eighth of the work instead of every eighth item, so
// that the bytes an XCD reads form one stretch of each plane (its address translations and its L2 cover an eighth
// of the pages instead of all of them): the grid is padded to a multiple of eight workgroups, workgroup L takes
// item xcd_work_index(L, grid) and leaves at once when that is not below the number of items.
constexpr int kXcds = 8;
inline unsigned xcd_grid(size_t items) { return (unsigned)((items + kXcds - 1) / kXcds * kXcds); }

// ------------------------------------------------------------------ device helpers
#if defined(__HIPCC__)
__device__ __forceinline__ int xcd_work_index(int L, int nwg) { return (L % kXcds) * (nwg / kXcds) + L / kXcds; }

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float half_bits_to_float(uint32_t h)
{
    return (float)__builtin_bit_cast(_Float16, (uint16_t)h);   // exact
}
__device__ __forceinline__ uint32_t float_bits(float f) { return __builtin_bit_cast(uint32_t, f); }
// takes the word BY VALUE: __builtin_bit_cast applied directly to a vector component (w.y) reads component 0
__device__ __forceinline__ float bits_float(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ int float_exp_field(float f) { return (int)((float_bits(f) >> 23) & 0xFFu); }

// smallest level keeping at least m mantissa bits (2 / 6 / 10 kept at level 0 / 1 / 2)
__device__ __forceinline__ int level_for_mantissa_bits(int m) { return m <= 2 ? 0 : (m <= 6 ? 1 : 2); }

// Fill words for nibble planes that are not read ("Dynamic Quantization": the bits not read are 100...):
// level 0: MID nibble = 8, LO nibble = 0;  level 1: MID read, LO nibble = 8.
constexpr uint32_t kFill8 = 0x88888888u;

// Assemble eight fp16 values from their planes.  H0, H1: the eight HI bytes (element i in byte i%4 of
// H[i/4]); M, L: the eight MID / LO nibbles (element 2i in the low nibble of byte i).  Result: p[0] =
// elements (0,2), p[1] = (1,3), p[2] = (4,6), p[3] = (5,7), first of the pair in the low half.
__device__ __forceinline__ void assemble8(uint32_t H0, uint32_t H1, uint32_t M, uint32_t L, uint32_t (&p)[4])
{
    const uint32_t ev = ((M << 4) & 0xF0F0F0F0u) | (L & 0x0F0F0F0Fu);   // low bytes of elements 0,2,4,6
    const uint32_t od = (M & 0xF0F0F0F0u) | ((L >> 4) & 0x0F0F0F0Fu);   // low bytes of elements 1,3,5,7
    // v_perm_b32: result byte i = byte sel[i] of the pool {src0 (bytes 7..4), src1 (bytes 3..0)}
    p[0] = __builtin_amdgcn_perm(H0, ev, 0x06010400u);
    p[1] = __builtin_amdgcn_perm(H0, od, 0x07010500u);
    p[2] = __builtin_amdgcn_perm(H1, ev, 0x06030402u);
    p[3] = __builtin_amdgcn_perm(H1, od, 0x07030502u);
}

// Raw buffer loads (the hardware range check makes predication free): a load whose byte offset is at or
// beyond the buffer's size returns zero and fetches nothing, so "do not read this plane" is an offset of
// kSkip instead of a branch, and every load of a loop can be issued unconditionally and early.
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
constexpr uint32_t kSkip = 0x80000000u;
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);   // raw, 32-bit format
}
__device__ __forceinline__ uint32_t buf_load_b32(__amdgpu_buffer_rsrc_t r, uint32_t off)
{
    return __builtin_amdgcn_raw_buffer_load_b32(r, off, 0, 0);
}
__device__ __forceinline__ u32x2_t buf_load_b64(__amdgpu_buffer_rsrc_t r, uint32_t off)
{
    return __builtin_amdgcn_raw_buffer_load_b64(r, off, 0, 0);
}
__device__ __forceinline__ u32x4_t buf_load_b128(__amdgpu_buffer_rsrc_t r, uint32_t off)
{
    return __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, 0);
}

// The same with the non-temporal hint: cache bytes that are read once per step stream through L2 without pushing out
// what is read again (the logits between the passes, the lines an appended token is stored into).
constexpr int kAuxNt = 2;
__device__ __forceinline__ u32x2_t buf_load_b64_nt(__amdgpu_buffer_rsrc_t r, uint32_t off)
{
    return __builtin_amdgcn_raw_buffer_load_b64(r, off, 0, kAuxNt);
}
__device__ __forceinline__ u32x4_t buf_load_b128_nt(__amdgpu_buffer_rsrc_t r, uint32_t off)
{
    return __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, kAuxNt);
}

// Data handed from one workgroup to another INSIDE a kernel (the chunk partials of the V kernel and the slab
// partials of the weight GEMV, to the workgroup that combines them).  The L2 caches of the eight XCDs are not
// coherent with each other, and a device-scope fence writes back / invalidates a whole L2, which costs far
// more than the data is worth.  So these few words are moved with device-scope relaxed accesses (sc1: written
// through to memory, read from memory), the producer waits for its stores to be acknowledged before it takes
// its ticket with a device-scope atomic, and the consumer issues its loads after it has seen the last ticket.
constexpr int kAuxSc1 = 16;   // cache policy bit of raw buffer accesses: device (agent) scope
__device__ __forceinline__ void store_agent(float* p, float v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float load_agent(const float* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store_agent(int32_t* p, int32_t v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ int32_t load_agent(const int32_t* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// all of this wave's earlier stores have been acknowledged (and the compiler keeps them above this point)
__device__ __forceinline__ void stores_done()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0);
}
__device__ __forceinline__ int take_ticket(int32_t* counter)
{
    return __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Variant of assemble8 taking the fill for unread bits as a per-byte constant OR-ed into the low bytes:
// level 0 -> 0x80808080 (with M = L = 0), level 1 -> 0x08080808 (with L = 0), level 2 -> 0.
// (a & mask) | (b & ~mask) in one instruction (the compiler settles for two ANDs and a three-way OR otherwise)
__device__ __forceinline__ uint32_t bit_select(uint32_t mask, uint32_t a, uint32_t b)
{
    uint32_t r;
    asm("v_bfi_b32 %0, %1, %2, %3" : "=v"(r) : "s"(mask), "v"(a), "v"(b));
    return r;
}
__device__ __forceinline__ void assemble8_fill(uint32_t H0, uint32_t H1, uint32_t M, uint32_t L, uint32_t fill,
                                               uint32_t (&p)[4])
{
    const uint32_t ev = bit_select(0xF0F0F0F0u, M << 4, L) | fill;
    const uint32_t od = bit_select(0xF0F0F0F0u, M, L >> 4) | fill;
    p[0] = __builtin_amdgcn_perm(H0, ev, 0x06010400u);
    p[1] = __builtin_amdgcn_perm(H0, od, 0x07010500u);
    p[2] = __builtin_amdgcn_perm(H1, ev, 0x06030402u);
    p[3] = __builtin_amdgcn_perm(H1, od, 0x07030502u);
}
__device__ __forceinline__ uint32_t fill_for_level(int lv) { return lv == 0 ? 0x80808080u : (lv == 1 ? 0x08080808u : 0u); }

__device__ __forceinline__ float lo_half(uint32_t p) { return (float)__builtin_bit_cast(half2_t, p).x; }
__device__ __forceinline__ float hi_half(uint32_t p) { return (float)__builtin_bit_cast(half2_t, p).y; }

// Score exponent of a logit ("Quantization of V-Cache": the scores span many orders of magnitude):
// x = (l - M) * c in two separately rounded fp32 operations, a = max(floor(x), -64).
__device__ __forceinline__ float score_x(float l, float M, float c)
{
    const float diff = l - M;
    return diff * c;            // the file is compiled with -ffp-contract=off: no fusion
}
__device__ __forceinline__ int score_a(float x)
{
    const float fl = floorf(x);
    return fl < (float)kAMin ? kAMin : (int)fl;
}

// Inclusive prefix sum over the 64 lanes of a wave in the vector ALU (six data-parallel-primitive steps: shifts by
// 1, 2, 4, 8 inside the rows of 16 lanes, then lane 15 of a row added to the next row, then lane 31 to the upper
// half); a lane without a source adds zero.
__device__ __forceinline__ int wave_scan_add(int v)
{
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xF, 0xF, false);   // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xF, 0xF, false);   // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xF, 0xF, false);   // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xF, 0xF, false);   // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xA, 0xF, false);   // row_bcast:15 into rows 1 and 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xC, 0xF, false);   // row_bcast:31 into rows 2 and 3
    return v;
}
// value of lane `l` (wave-uniform index) in every lane
__device__ __forceinline__ int wave_read(int v, int l) { return __builtin_amdgcn_readlane(v, l); }

// maximum over the 64 lanes of a wave, in every lane: the steps of wave_scan_add with max (a lane without a source
// keeps its value), then lane 63 holds the maximum of all
__device__ __forceinline__ float wave_max(float v)
{
    auto step = [](float x, int ctrl_sel) {
        const int xi = __builtin_bit_cast(int, x);
        int yi;
        switch (ctrl_sel) {
            case 0: yi = __builtin_amdgcn_update_dpp(xi, xi, 0x111, 0xF, 0xF, false); break;
            case 1: yi = __builtin_amdgcn_update_dpp(xi, xi, 0x112, 0xF, 0xF, false); break;
            case 2: yi = __builtin_amdgcn_update_dpp(xi, xi, 0x114, 0xF, 0xF, false); break;
            case 3: yi = __builtin_amdgcn_update_dpp(xi, xi, 0x118, 0xF, 0xF, false); break;
            case 4: yi = __builtin_amdgcn_update_dpp(xi, xi, 0x142, 0xA, 0xF, false); break;
            default: yi = __builtin_amdgcn_update_dpp(xi, xi, 0x143, 0xC, 0xF, false); break;
        }
        return fmaxf(x, __builtin_bit_cast(float, yi));
    };
#pragma unroll
    for (int k = 0; k < 6; ++k) v = step(v, k);
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

// the same for integers
__device__ __forceinline__ int wave_max_int(int v)
{
    v = max(v, __builtin_amdgcn_update_dpp(v, v, 0x111, 0xF, 0xF, false));
    v = max(v, __builtin_amdgcn_update_dpp(v, v, 0x112, 0xF, 0xF, false));
    v = max(v, __builtin_amdgcn_update_dpp(v, v, 0x114, 0xF, 0xF, false));
    v = max(v, __builtin_amdgcn_update_dpp(v, v, 0x118, 0xF, 0xF, false));
    v = max(v, __builtin_amdgcn_update_dpp(v, v, 0x142, 0xA, 0xF, false));
    v = max(v, __builtin_amdgcn_update_dpp(v, v, 0x143, 0xC, 0xF, false));
    return __builtin_amdgcn_readlane(v, 63);
}

#endif  // __HIPCC__
}  // namespace akv
