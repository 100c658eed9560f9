// C ABI of the library (declared in include/akv.h): argument checks, workspace carving, launches.
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <vector>

#include "akv_common.h"

namespace {

thread_local char g_err[256] = "";

constexpr auto fail = &akv::fail_msg;   // one error record for every entry point of the library

bool aligned16(const void* p) { return reinterpret_cast<uintptr_t>(p) % 16 == 0; }

bool shape_ok(const akv_shape& s)
{
    return s.B > 0 && s.Hq > 0 && s.Hkv > 0 && s.D == akv::kD && s.Hq % s.Hkv == 0 && s.Hq / s.Hkv <= akv::kMaxG &&
           ((s.Hq / s.Hkv) & (s.Hq / s.Hkv - 1)) == 0 && s.Ncap > 0 && s.Ncap % AKV_TB == 0 && s.Ncap <= (1 << 22) &&
           size_t(s.B) * s.Hq * size_t(s.Ncap) < (size_t(1) << 40);
}

akv_status check_cache(const akv_cache* c)
{
    if (!c) return fail(AKV_EINVAL, "cache is NULL");
    if (!shape_ok(c->shape))
        return fail(AKV_EINVAL, "bad shape: B=%d Hq=%d Hkv=%d D=%d Ncap=%d (need D=128, Hq/Hkv a power of two <= 8, Ncap %% 256 == 0)",
                    c->shape.B, c->shape.Hq, c->shape.Hkv, c->shape.D, c->shape.Ncap);
    if (!c->k_hi || !c->k_mid || !c->k_lo || !c->v_hi || !c->v_mid || !c->v_lo || !c->colmax || !c->lens || !c->flags)
        return fail(AKV_EINVAL, "cache has a NULL plane / colmax / lens / flags pointer");
    if (!aligned16(c->k_hi) || !aligned16(c->k_mid) || !aligned16(c->k_lo) || !aligned16(c->v_hi) || !aligned16(c->v_mid) ||
        !aligned16(c->v_lo) || !aligned16(c->colmax) || reinterpret_cast<uintptr_t>(c->lens) % 4 || reinterpret_cast<uintptr_t>(c->flags) % 4)
        return fail(AKV_EINVAL, "cache planes and colmax must be 16-byte aligned, lens and flags 4-byte aligned");
    return AKV_OK;
}

akv_status hip_fail(hipError_t e, const char* what)
{
    return fail(AKV_EHIP, "%s: %s", what, hipGetErrorString(e));
}

}  // namespace

namespace akv {
akv_status fail_msg(akv_status st, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return st;
}
int compute_units()
{
    static int cus = 0;
    if (cus == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0) cus = n;
        else cus = 256;
    }
    return cus;
}
}  // namespace akv

extern "C" {

int akv_version(void) { return 101; }

const char* akv_last_error(void) { return g_err; }

akv_status akv_layout_sizes(const akv_shape* shape, akv_sizes* out)
{
    if (!shape || !out) return fail(AKV_EINVAL, "NULL argument");
    if (!shape_ok(*shape))
        return fail(AKV_EINVAL, "bad shape: B=%d Hq=%d Hkv=%d D=%d Ncap=%d (need D=128, Hq/Hkv a power of two <= 8, Ncap %% 256 == 0)",
                    shape->B, shape->Hq, shape->Hkv, shape->D, shape->Ncap);
    const size_t e = size_t(shape->B) * shape->Hkv * size_t(shape->Ncap) * shape->D;   // elements of K (and of V)
    out->k_hi = e; out->k_mid = e / 2; out->k_lo = e / 2;
    out->v_hi = e; out->v_mid = e / 2; out->v_lo = e / 2;
    out->colmax = size_t(shape->B) * shape->Hkv * shape->D * sizeof(uint16_t);
    out->lens = size_t(shape->B) * sizeof(int32_t);
    out->flags = (AKV_NFLAGS + size_t(shape->B)) * sizeof(int32_t);
    out->workspace = akv::ws_layout(*shape).total;
    out->fp16_workspace = akv::fp16_workspace_bytes(*shape);
    return AKV_OK;
}

akv_status akv_cache_reset(const akv_cache* cache, void* stream)
{
    if (akv_status st = check_cache(cache)) return st;
    akv_sizes sz;
    akv_layout_sizes(&cache->shape, &sz);
    hipStream_t s = static_cast<hipStream_t>(stream);
    struct { void* p; size_t n; } bufs[] = {
        {cache->k_hi, sz.k_hi}, {cache->k_mid, sz.k_mid}, {cache->k_lo, sz.k_lo}, {cache->v_hi, sz.v_hi},
        {cache->v_mid, sz.v_mid}, {cache->v_lo, sz.v_lo}, {cache->colmax, sz.colmax}, {cache->lens, sz.lens},
        {cache->flags, sz.flags}};
    for (auto& bf : bufs) {
        if (hipError_t e = akv::launch_zero(bf.p, bf.n, s)) return hip_fail(e, "zero launch");
    }
    return AKV_OK;
}

akv_status akv_workspace_init(const akv_shape* shape, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!shape || !shape_ok(*shape)) return fail(AKV_EINVAL, "bad shape");
    const akv::WsLayout w = akv::ws_layout(*shape);
    if (!workspace || workspace_bytes < w.total)
        return fail(AKV_EWORKSPACE, "workspace of %zu bytes given, %zu needed", workspace_bytes, w.total);
    if (reinterpret_cast<uintptr_t>(workspace) % 256) return fail(AKV_EWORKSPACE, "workspace is not 256-byte aligned");
    if (hipError_t e = akv::launch_zero(static_cast<char*>(workspace) + w.control, akv::align256(w.control_bytes),
                                        static_cast<hipStream_t>(stream)))
        return hip_fail(e, "zero launch");
    return AKV_OK;
}

akv_status akv_append(const akv_cache* cache, const uint16_t* k_new, const uint16_t* v_new, const int32_t* n_new,
                      int32_t n, void* stream)
{
    if (akv_status st = check_cache(cache)) return st;
    if (n < 0 || n > cache->shape.Ncap) return fail(AKV_EINVAL, "n = %d out of range 0..Ncap", n);
    if (n > 0 && (!k_new || !v_new)) return fail(AKV_EINVAL, "k_new / v_new is NULL");
    if (!aligned16(k_new) || !aligned16(v_new)) return fail(AKV_EINVAL, "k_new / v_new must be 16-byte aligned");
    if (hipError_t e = akv::launch_append(*cache, k_new, v_new, n_new, n, static_cast<hipStream_t>(stream)))
        return hip_fail(e, "append launch");
    return AKV_OK;
}

akv_status akv_check_capacity_sync(const akv_cache* cache, int32_t n, void* stream)
{
    if (akv_status st = check_cache(cache)) return st;
    if (n < 0) return fail(AKV_EINVAL, "n = %d is negative", n);
    const int B = cache->shape.B;
    std::vector<int32_t> lens(B);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (hipError_t e = hipMemcpyAsync(lens.data(), cache->lens, size_t(B) * sizeof(int32_t), hipMemcpyDeviceToHost, s)) return hip_fail(e, "hipMemcpyAsync");
    if (hipError_t e = hipStreamSynchronize(s)) return hip_fail(e, "hipStreamSynchronize");
    for (int b = 0; b < B; ++b)
        if (long(lens[b]) + n > cache->shape.Ncap)
            return fail(AKV_ECAPACITY, "sequence %d holds %d tokens: %d more exceed the capacity of %d", b, lens[b], n, cache->shape.Ncap);
    return AKV_OK;
}

akv_status akv_stream_read(const void* buf, size_t bytes, uint32_t* sink, void* stream)
{
    if (!buf || !sink) return fail(AKV_EINVAL, "buf / sink is NULL");
    if ((reinterpret_cast<uintptr_t>(buf) & 15) || (bytes & 15)) return fail(AKV_EINVAL, "buf and bytes must be multiples of 16");
    if (hipError_t e = akv::launch_stream_read(buf, bytes, sink, static_cast<hipStream_t>(stream)))
        return hip_fail(e, "stream read launch");
    return AKV_OK;
}

akv_status akv_unpack(const akv_cache* cache, uint16_t* k_out, uint16_t* v_out, void* stream)
{
    if (akv_status st = check_cache(cache)) return st;
    if (!k_out && !v_out) return AKV_OK;
    if (!aligned16(k_out) || !aligned16(v_out)) return fail(AKV_EINVAL, "k_out / v_out must be 16-byte aligned");
    if (hipError_t e = akv::launch_unpack(*cache, k_out, v_out, static_cast<hipStream_t>(stream)))
        return hip_fail(e, "unpack launch");
    return AKV_OK;
}

}  // extern "C"

// ---- the scratch of akv_decode_attention_static: one device array per GPU, never allocated or freed ------------
// In host code the array's name is only a handle: its device address is looked up per device and kept.
static __device__ __align__(256) unsigned char akv_static_scratch[AKV_STATIC_SCRATCH_BYTES];

namespace {

using akv::compute_units;

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of the static scratch array on the current device; on the first call on a device its control block
// is zeroed by a fill kernel on `s` (ordered in front of the decode kernels that follow on the same stream).
// Returns nullptr after recording the error text.
void* static_scratch_for_current_device(hipStream_t s)
{
    int dev = -1;
    if (hipError_t e = hipGetDevice(&dev)) { hip_fail(e, "hipGetDevice"); return nullptr; }
    if (dev < 0 || dev >= kMaxDevices) { fail(AKV_EHIP, "device ordinal %d out of range", dev); return nullptr; }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(akv_static_scratch))) { hip_fail(e, "hipGetSymbolAddress"); return nullptr; }
        if (!ptr) { fail(AKV_EHIP, "hipGetSymbolAddress returned a null address"); return nullptr; }
        if (hipError_t e = akv::launch_zero(ptr, akv::kCtlReserve, s)) { hip_fail(e, "zero launch"); return nullptr; }
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

// Head-per-workgroup or token-split kernels, when the caller leaves the choice to the library.  One head kernel
// workgroup occupies a compute unit, so `pairs` (sequence, KV head) pairs run in ceil(pairs / CUs) rounds of equal
// length: the path pays when there is one round and it is nearly full, or when the sequences are so short that the
// single launch outweighs idle units; for single query heads also at two nearly full rounds, as long as the logits of
// a pair fit its LDS (the token-split kernels write theirs to memory, and written bytes cost several times what read
// bytes cost).  The thresholds are where the two paths crossed when timed over pairs = 64..1024, lengths 1024..12288
// and group sizes 1, 2, 4 on MI355X.
bool head_path_pays(long pairs, int G, int max_len)
{
    const long cus = compute_units();
    if (pairs > cus) return G == 1 && pairs <= 2 * cus && double(pairs) / double(2 * cus) >= 0.85 && max_len <= 8192;
    if (max_len <= (G == 1 ? 2048 : 1024)) return true;
    const double fill = double(pairs) / double(cus);
    if (G == 1) return (max_len <= 8192 && fill >= 0.72) || (max_len <= 12288 && fill >= 0.85);
    if (G == 2) return max_len <= 8192 && fill >= 0.9;
    return (max_len <= 2048 && fill >= 0.6) || (max_len <= 4096 && fill >= 0.85) || (max_len <= 6144 && fill >= 0.97);
}

// decode attention, optionally preceded by the append of one token per sequence (k_new, v_new: [B][Hkv][D])
// static_scratch: the workspace is the library's own device array (akv_decode_attention_static)
akv_status decode_impl(const akv_cache* cache, const uint16_t* k_new, const uint16_t* v_new, const uint16_t* q, void* out,
                       const akv_params* params, void* workspace, size_t workspace_bytes, void* stream,
                       bool static_scratch = false)
{
    if (akv_status st = check_cache(cache)) return st;
    if (!q || !out) return fail(AKV_EINVAL, "q / out is NULL");
    if (!aligned16(q) || !aligned16(out) || !aligned16(k_new) || !aligned16(v_new))
        return fail(AKV_EINVAL, "q, out, k_new and v_new must be 16-byte aligned");
    akv_params p;
    std::memset(&p, 0, sizeof p);
    p.force_level = -1;
    if (params) p = *params;
    if (p.topk == 0) p.topk = 32;
    if (p.topk < 1 || p.topk > AKV_MAX_TOPK) return fail(AKV_EINVAL, "topk = %d out of range 1..%d", p.topk, AKV_MAX_TOPK);
    if (p.guard_bits < 0 || p.guard_bits > 12) return fail(AKV_EINVAL, "guard_bits = %d out of range 0..12", p.guard_bits);
    if (p.force_level < -1 || p.force_level > 2) return fail(AKV_EINVAL, "force_level = %d out of range -1..2", p.force_level);
    if (p.out_dtype != 0 && p.out_dtype != 1) return fail(AKV_EINVAL, "out_dtype = %d is neither 0 (f32) nor 1 (f16)", p.out_dtype);
    if (p.max_len < 0 || p.max_len > cache->shape.Ncap) return fail(AKV_EINVAL, "max_len = %d out of range 0..Ncap", p.max_len);
    if (!(p.scale == p.scale) || std::isinf(p.scale)) return fail(AKV_EINVAL, "scale is not finite");
    const akv::WsLayout w = akv::ws_layout(cache->shape, static_scratch);
    if (static_scratch) {
        if (w.total > AKV_STATIC_SCRATCH_BYTES || w.control_bytes > akv::kCtlReserve)
            return fail(AKV_EWORKSPACE, "this shape needs %zu bytes of scratch (%zu of control words); the static array holds %zu (%zu): "
                        "use akv_decode_attention with a workspace of the caller's", w.total, w.control_bytes,
                        size_t(AKV_STATIC_SCRATCH_BYTES), akv::kCtlReserve);
        hipStream_t s0 = static_cast<hipStream_t>(stream);
        workspace = static_scratch_for_current_device(s0);
        if (!workspace) return AKV_EHIP;   // the text has been recorded
        workspace_bytes = AKV_STATIC_SCRATCH_BYTES;
    }
    if (!workspace || workspace_bytes < w.total)
        return fail(AKV_EWORKSPACE, "workspace of %zu bytes given, %zu needed", workspace_bytes, w.total);
    if (reinterpret_cast<uintptr_t>(workspace) % 256) return fail(AKV_EWORKSPACE, "workspace is not 256-byte aligned");
    if (p.stats && reinterpret_cast<uintptr_t>(p.stats) % 8) return fail(AKV_EINVAL, "stats must be 8-byte aligned");

    akv::DecodeArgs a;
    std::memset(&a, 0, sizeof a);
    a.s = cache->shape;
    a.k_hi = cache->k_hi; a.k_mid = cache->k_mid; a.k_lo = cache->k_lo;
    a.v_hi = cache->v_hi; a.v_mid = cache->v_mid; a.v_lo = cache->v_lo;
    a.colmax = cache->colmax; a.lens = cache->lens; a.q = q; a.out = out;
    a.flags = cache->flags;
    const double scale = p.scale > 0.0f ? (double)p.scale : 1.0 / std::sqrt((double)a.s.D);
    a.c = (float)(scale * 1.4426950408889634);
    a.topk = p.topk; a.guard_bits = p.guard_bits; a.force_level = p.force_level; a.out_dtype = p.out_dtype;
    a.max_len = p.max_len > 0 ? p.max_len : a.s.Ncap;
    {   // V kernel of the token-split path: one round of workgroups that fills the device -- the tokens of a
        // (sequence, KV head) pair are cut into as many chunks as there are resident workgroups per pair, so that
        // the fixed costs per workgroup (Rule 2 constants, pipeline start, partial results) are paid once per slot
        const int cus = compute_units();
        const int G = a.s.Hq / a.s.Hkv;
        const int per_cu = akv::split_v_workgroups_per_cu(G);
        const long pairs = long(a.s.B) * a.s.Hkv;
        const long per_pair = std::max(1L, long(cus) * per_cu / pairs);
        long chunk = (a.max_len + per_pair - 1) / per_pair;
        chunk = (chunk + 63) / 64 * 64;                       // whole batches of rows for every wave
        a.vchunk = int(std::max(long(akv::kVChunk), chunk));
    }
    char* ws = static_cast<char*>(workspace);
    a.logits = reinterpret_cast<float*>(ws + w.logits);
    a.tilemax = reinterpret_cast<float*>(ws + w.tilemax);
    a.M = reinterpret_cast<float*>(ws + w.M);
    a.hist = reinterpret_cast<int32_t*>(ws + w.hist);
    a.cand_sel = reinterpret_cast<int32_t*>(ws + w.cand_sel);
    a.cand_phat = reinterpret_cast<float*>(ws + w.cand_phat);
    a.Ehat = reinterpret_cast<int32_t*>(ws + w.Ehat);
    a.partO = reinterpret_cast<float*>(ws + w.partO);
    a.partZ = reinterpret_cast<float*>(ws + w.partZ);
    a.kcount = reinterpret_cast<int32_t*>(ws + w.control);
    a.vcount = a.kcount + size_t(a.s.B) * a.s.Hkv;
    a.stats = p.stats;
    if (p.dbg) {
        a.dbg = *p.dbg;
        if (a.dbg.logits) a.logits = a.dbg.logits;   // same shape: the pass writes the export directly
    }
    if (p.path < 0 || p.path > 2) return fail(AKV_EINVAL, "path = %d out of range 0..2", p.path);
    if (p.path == 1 && !akv::head_path_supported(a.s))
        return fail(AKV_EINVAL, "path 1 (head per workgroup) needs Hq/Hkv <= 4");
    const bool head_path = p.path == 1 || (p.path == 0 && akv::head_path_supported(a.s) &&
                                           head_path_pays(long(a.s.B) * a.s.Hkv, a.s.Hq / a.s.Hkv, a.max_len));
    hipStream_t s = static_cast<hipStream_t>(stream);
    auto ev = [&](int i) -> hipEvent_t { return p.events ? static_cast<hipEvent_t>(p.events[i]) : nullptr; };
    if (p.events)
        if (hipError_t e = hipEventRecord(ev(0), s)) return hip_fail(e, "hipEventRecord");
    if (head_path) {
        if (p.events)
            for (int i = 1; i < 4; ++i)
                if (hipError_t e = hipEventRecord(ev(i), s)) return hip_fail(e, "hipEventRecord");
        a.k_new = k_new;   // the head kernel stores the new token itself
        a.v_new = v_new;
        if (hipError_t e = akv::launch_decode_head(a, s)) return hip_fail(e, "decode (head path) launch");
    } else {
        if (k_new)
            if (hipError_t e = akv::launch_append(*cache, k_new, v_new, nullptr, 1, s)) return hip_fail(e, "append launch");
        if (p.events)
            if (hipError_t e = hipEventRecord(ev(1), s)) return hip_fail(e, "hipEventRecord");
        if (hipError_t e = akv::launch_decode_split(a, s, ev(2), ev(3))) return hip_fail(e, "decode (split path) launch");
    }
    if (p.events)
        if (hipError_t e = hipEventRecord(ev(4), s)) return hip_fail(e, "hipEventRecord");
    return AKV_OK;
}

}  // namespace

extern "C" {

akv_status akv_decode_attention(const akv_cache* cache, const uint16_t* q, void* out, const akv_params* params,
                                void* workspace, size_t workspace_bytes, void* stream)
{
    return decode_impl(cache, nullptr, nullptr, q, out, params, workspace, workspace_bytes, stream);
}

int32_t akv_decode_path(const akv_shape* shape, int32_t max_len)
{
    if (!shape || !shape_ok(*shape) || max_len < 0 || max_len > shape->Ncap) return 0;
    const int ml = max_len > 0 ? max_len : shape->Ncap;
    if (!(akv::head_path_supported(*shape) && head_path_pays(long(shape->B) * shape->Hkv, shape->Hq / shape->Hkv, ml))) return 2;
    return akv::head_logits_in_lds(*shape, ml) ? 3 : 1;
}

akv_status akv_decode_attention_static(const akv_cache* cache, const uint16_t* q, void* out, const akv_params* params,
                                       void* stream)
{
    return decode_impl(cache, nullptr, nullptr, q, out, params, nullptr, 0, stream, true);
}

akv_status akv_append_decode_attention(const akv_cache* cache, const uint16_t* k_new, const uint16_t* v_new,
                                       const uint16_t* q, void* out, const akv_params* params, void* workspace,
                                       size_t workspace_bytes, void* stream)
{
    if (!k_new || !v_new) return fail(AKV_EINVAL, "k_new / v_new is NULL");
    return decode_impl(cache, k_new, v_new, q, out, params, workspace, workspace_bytes, stream);
}

akv_status akv_fp16_decode_attention(const akv_shape* shape, const uint16_t* k, const uint16_t* v, const int32_t* lens,
                                     const uint16_t* q, void* out, float scale, int32_t out_dtype, int32_t max_len,
                                     void* workspace, size_t workspace_bytes, void* stream)
{
    if (!shape || !shape_ok(*shape)) return fail(AKV_EINVAL, "bad shape");
    if (!k || !v || !lens || !q || !out) return fail(AKV_EINVAL, "NULL pointer argument");
    if (!aligned16(k) || !aligned16(v) || !aligned16(q) || !aligned16(out)) return fail(AKV_EINVAL, "k, v, q and out must be 16-byte aligned");
    if (out_dtype != 0 && out_dtype != 1) return fail(AKV_EINVAL, "out_dtype = %d is neither 0 (f32) nor 1 (f16)", out_dtype);
    if (max_len < 0 || max_len > shape->Ncap) return fail(AKV_EINVAL, "max_len = %d out of range 0..Ncap", max_len);
    const size_t need = akv::fp16_workspace_bytes(*shape);
    if (!workspace || workspace_bytes < need)
        return fail(AKV_EWORKSPACE, "workspace of %zu bytes given, %zu needed", workspace_bytes, need);
    if (reinterpret_cast<uintptr_t>(workspace) % 256) return fail(AKV_EWORKSPACE, "workspace is not 256-byte aligned");
    const float sc = scale > 0.0f ? scale : (float)(1.0 / std::sqrt((double)shape->D));
    if (hipError_t e = akv::launch_fp16(*shape, k, v, lens, q, out, sc, out_dtype, max_len > 0 ? max_len : shape->Ncap,
                                        workspace, static_cast<hipStream_t>(stream)))
        return hip_fail(e, "fp16 attention launch");
    return AKV_OK;
}

}  // extern "C"
