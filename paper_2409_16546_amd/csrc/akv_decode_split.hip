// Decode attention, token-split path: the tokens of every (sequence, KV head) are spread over many
// workgroups (long contexts, few heads).  Four kernels:
//   K kernel          Rule 1 levels + q.K~, one 256-token block per wave;
//   slice kernel      max, score exponents, their histogram and the local top-k candidates per 1024-token slice;
//   selection kernel  one workgroup per (sequence, KV head): the top-k from the slices' histograms and candidates,
//                     O_est and the result exponents;
//   V kernel          Rule 2 + S.V~ over chunks of tokens; the workgroup that finishes last combines the chunks.
// Sections "Quantization of K-Cache", "Quantization of V-Cache", "Runtime of AlignedKV".
#include <type_traits>
#include "akv_common.h"
#include "akv_k_tile.h"
#include "akv_mid_step.h"
#include "akv_v_rows.h"

namespace akv {

// K kernel: workgroup = kKWaves waves = one slice of kMidSlice tokens of one (sequence, KV head); a wave walks one
// 256-token block and leaves its logits and its block maximum in the workspace.
template <int G>
__global__ __launch_bounds__(64 * kKWaves) void split_k_kernel(DecodeArgs a)
{
    __shared__ __align__(16) uint8_t kstage[kKWaves][kKStage];
    __shared__ KShared<G> ks;

    const int h = blockIdx.y, b = blockIdx.z;
    const int lane = threadIdx.x & 63;
    const int Hq = a.s.Hq, Ncap = a.s.Ncap, NB = Ncap / kTB;
    const int len = min(min(a.lens[b], Ncap), a.max_len);   // a hint below the true length: the tokens past it are left out, consistently in all four kernels
    const int wave_u = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    const int blk = blockIdx.x * kKWaves + wave_u;
    if (blockIdx.x * kMidSlice >= len) return;   // whole workgroup beyond the sequence (uniform)

    if (blockIdx.x == 0 && h == 0 && threadIdx.x == 0 && min(a.lens[b], Ncap) > a.max_len) atomicAdd(&a.flags[AKV_FLAG_MAXLEN], 1);
    k_levels<G>(a, b, h, ks, blockIdx.x == 0, len);
    if (blk * kTB < len) {                       // else this wave's block is beyond the sequence
        float tm[G];
        const u32x4_t zero4 = {0u, 0u, 0u, 0u};
        const u32x4_t none[6] = {zero4, zero4, zero4, zero4, zero4, zero4};
        float lg[G][4];
        k_tile<G>(a, b, h, blk, len, ks, 0, tm, none, false, lg, &kstage[wave_u][0]);
        if (lane == 0)
#pragma unroll
            for (int g = 0; g < G; ++g) a.tilemax[(size_t(b) * Hq + size_t(h) * G + g) * NB + blk] = tm[g];
    }
}

// Mid step in two kernels.
// Slice kernel: workgroup = 256 threads = one slice of kMidSlice tokens of one (sequence, KV head).  Every workgroup
// derives the global max logit from the block maxima and, per query head (a wave each), (1) builds the histogram of
// score exponents of its slice and leaves it in the workspace as running sums over the buckets, (2) selects the
// approximate top-k' of its own slice -- a superset of what the whole sequence can select from it, because the
// cut bucket of the sequence is never later than the slice's own -- and leaves those candidates (token, bucket,
// weight, in token order) in the workspace.  Little LDS, so that every slice of a long batch is resident at once.
// Selection kernel: one workgroup per (sequence, KV head); each query head of the group goes to one of its waves:
// the wave adds the slices' running sums (the first bucket where the total reaches k' is the cut), reads two words
// per slice to learn how many selected tokens precede each slice and which slices hold any, and takes the
// selection out of those slices' candidate lists (lane = candidate, ballots give the order); then all threads
// compute O_est and the result exponents -- the V rows of all query heads are asked for before the first is used.
// Everything that grows with the length of the sequence is spread over the slices; every dependent step of the
// selection is one round trip to memory.
template <int G>
__global__ __launch_bounds__(256, (G <= 4 ? 8 : 4)) void split_slice_kernel(DecodeArgs a)   // every slice of a long batch resident at once
{
    constexpr int NT = 256, kWaves = NT / 64;
    static_assert(kMidSlice == NT * 4, "a thread owns four tokens of the slice");
    __shared__ float red_s[G][kWaves];
    __shared__ float M_s[G];
    __shared__ int cntw_s[kWaves][kBuckets + 1];

    const int slice = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int Hq = a.s.Hq, Ncap = a.s.Ncap, NB = Ncap / kTB;
    const int S = (Ncap + kMidSlice - 1) / kMidSlice;   // slices per query head in the workspace
    const int len = min(min(a.lens[b], Ncap), a.max_len);   // a hint below the true length: the tokens past it are left out, consistently in all four kernels
    if (slice * kMidSlice >= len) return;   // uniform; also every empty sequence
    const int nblk = (len + kTB - 1) / kTB;
    const int kk = a.topk < len ? a.topk : len;

    // M = max over the block maxima (exact, order-free); the loads of all query heads of the group go out together
    float mg[G];
#pragma unroll
    for (int g = 0; g < G; ++g) mg[g] = tid < nblk ? a.tilemax[(size_t(b) * Hq + size_t(h) * G + g) * NB + tid] : -INFINITY;
    for (int i = tid + NT; i < nblk; i += NT)
#pragma unroll
        for (int g = 0; g < G; ++g) mg[g] = fmaxf(mg[g], a.tilemax[(size_t(b) * Hq + size_t(h) * G + g) * NB + i]);
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const float m = wave_max(mg[g]);
        if (lane == 0) red_s[g][wave] = m;
    }
    __syncthreads();
    if (tid < G) {
        float m = red_s[tid][0];
        for (int w = 1; w < kWaves; ++w) m = fmaxf(m, red_s[tid][w]);
        M_s[tid] = m;
        if (slice == 0) a.M[size_t(b) * Hq + size_t(h) * G + tid] = m;   // for the kernels that follow
    }
    __syncthreads();

    // ---- the slice: histogram and candidates, a wave per query head (lane -> 16 consecutive tokens; everything
    // below is wave-local: LDS serves a wave's accesses in order, no barrier) ------------------------------------
    {
        const int in_slice = min(len - slice * kMidSlice, kMidSlice);
        const int kloc = kk < in_slice ? kk : in_slice;   // candidates per query head
        const int t0 = slice * kMidSlice + lane * 16;
        for (int g = wave; g < G; g += kWaves) {
            const size_t hq = size_t(b) * Hq + size_t(h) * G + g;
            const __amdgpu_buffer_rsrc_t rs_lg = make_rsrc(a.logits + hq * Ncap, uint32_t(Ncap) * 4u);
            const float M = M_s[g];
            u32x4_t w[4];
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) w[q4] = __builtin_amdgcn_raw_buffer_load_b128(rs_lg, uint32_t(t0 + 4 * q4) * 4u, 0, 0);   // past Ncap: zeros
            int* hw = &cntw_s[wave][0];
            hw[lane] = 0;
            if (lane < 2) hw[64 + lane] = 0;
            float x[16];
            int j[16];   // bucket j = -a_t (1000 at or past len)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const float lv[4] = {bits_float(w[q4].x), bits_float(w[q4].y), bits_float(w[q4].z), bits_float(w[q4].w)};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int ii = 4 * q4 + i;
                    x[ii] = score_x(lv[i], M, a.c);
                    j[ii] = t0 + ii < len ? -score_a(x[ii]) : 1000;
                }
            }
            __builtin_amdgcn_wave_barrier();
            int n64 = 0;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                mid_hist_add(hw, j[i], n64);
                if (j[i] <= 64 && a.dbg.a) a.dbg.a[hq * Ncap + t0 + i] = (int8_t)(-j[i]);
            }
            mid_hist_flush(hw, n64);
            __builtin_amdgcn_wave_barrier();
            const int c = hw[lane];   // bucket `lane` of the slice's histogram
            int J, below;
            mid_find_cut(c, kloc, J, below);   // the slice's own cut: never earlier than the sequence's
            const int fromcut = kloc - below;
            {   // running sums over the buckets, for the workgroup that merges the slices
                const int incl = wave_scan_add(c);
                int32_t* dst = a.hist + (hq * S + slice) * kHistStride;
                dst[lane] = incl;                         // tokens in buckets 0..lane
                if (lane == 63) dst[64] = in_slice;       // all tokens of the slice
            }
            // the candidates in token order: tokens of each kind in lower lanes from five ballots per kind (one per
            // bit of the lane's count, at most 16)
            int c_lt = 0, c_eq = 0;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                c_lt += j[i] < J;
                c_eq += j[i] == J;
            }
            int n_lt = 0, n_eq = 0;
#pragma unroll
            for (int bit = 0; bit < 5; ++bit) {
                const uint64_t b_lt = __ballot((c_lt >> bit) & 1), b_eq = __ballot((c_eq >> bit) & 1);
                n_lt += __builtin_amdgcn_mbcnt_hi((uint32_t)(b_lt >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)b_lt, 0)) << bit;
                n_eq += __builtin_amdgcn_mbcnt_hi((uint32_t)(b_eq >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)b_eq, 0)) << bit;
            }
            const size_t base = (hq * S + slice) * AKV_MAX_TOPK;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const bool is_lt = j[i] < J, is_eq = j[i] == J;
                if (is_lt || (is_eq && n_eq < fromcut)) {
                    const int pos = n_lt + (n_eq < fromcut ? n_eq : fromcut);
                    const float fl = floorf(x[i]);
                    a.cand_sel[base + pos] = (t0 + i) | (j[i] << 24);
                    a.cand_phat[base + pos] = ldexpf(1.0f + (x[i] - fl), -j[i]);   // as mid_emit
                }
                n_lt += is_lt;
                n_eq += is_eq;
            }
            if (lane >= kloc) a.cand_sel[base + lane] = -1;   // no candidate
        }
    }
}

template <int G>
__global__ __launch_bounds__(256) void split_select_kernel(DecodeArgs a)
{
    constexpr int NT = 256, kWaves = NT / 64;
    static_assert(kWaves <= kMidSets, "a selection per wave");
    __shared__ MidShared ms;
    __shared__ int list_s[kWaves][AKV_MAX_TOPK], list_lt[kWaves][AKV_MAX_TOPK], list_eq[kWaves][AKV_MAX_TOPK];

    const int h = blockIdx.x, b = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int Hkv = a.s.Hkv, Hq = a.s.Hq, Ncap = a.s.Ncap;
    const int S = (Ncap + kMidSlice - 1) / kMidSlice;   // slices per query head in the workspace
    const int len = min(min(a.lens[b], Ncap), a.max_len);
    const size_t bh = size_t(b) * Hkv + h;
    if (len <= 0) return;   // uniform: an empty sequence has no selection (the V kernel writes its zeros)
    const int nsl = (len + kMidSlice - 1) / kMidSlice;
    const int kk = a.topk < len ? a.topk : len;

    int ehat = 32767;   // min over the group of the result exponent of channel tid (tid < D)
    for (int g0 = 0; g0 < G; g0 += kWaves) {
        const int g = g0 + wave;
        if (g < G) {   // wave-uniform: this wave collects the selection of query head g
            const size_t hq = size_t(b) * Hq + size_t(h) * G + g;
            const int32_t* hist = a.hist + hq * S * kHistStride;
            // running sums over the buckets, added over the slices: lane = bucket (0..63); 16 loads in flight
            int tot = 0;
            for (int s0 = 0; s0 < nsl; s0 += 16) {
                int v[16];
#pragma unroll
                for (int i = 0; i < 16; ++i) v[i] = s0 + i < nsl ? hist[(s0 + i) * kHistStride + lane] : 0;
#pragma unroll
                for (int i = 0; i < 16; ++i) tot += v[i];
            }
            const uint64_t reached = __ballot(tot >= kk);
            const int J = reached ? __builtin_ctzll(reached) : 64;   // bucket 64 is the cut only if none before it is
            const int below = J == 0 ? 0 : wave_read(tot, J - 1);
            const int fromcut = kk - below;
            // slices that hold selected tokens, with the number of tokens of each kind before them: lane = slice
            int nlist = 0, carry_lt = 0, carry_eq = 0;
            for (int s0 = 0; s0 < nsl; s0 += 64) {
                const int s = s0 + lane;
                int c_lt = 0, c_le = 0;
                if (s < nsl) {
                    if (J > 0) c_lt = hist[s * kHistStride + J - 1];
                    c_le = hist[s * kHistStride + J];
                }
                const int c_eq = c_le - c_lt;
                const int i_lt = wave_scan_add(c_lt), i_eq = wave_scan_add(c_eq);   // inclusive over the lanes
                const int p_lt = carry_lt + i_lt - c_lt, p_eq = carry_eq + i_eq - c_eq;   // exclusive prefixes
                const bool holds = c_lt > 0 || (c_eq > 0 && p_eq < fromcut);
                const uint64_t hb = __ballot(holds);   // at most kk such slices in all: each holds a selected token
                if (holds) {
                    const int at = nlist + __builtin_amdgcn_mbcnt_hi((uint32_t)(hb >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)hb, 0));
                    list_s[wave][at] = s;
                    list_lt[wave][at] = p_lt;
                    list_eq[wave][at] = p_eq;
                }
                nlist += __builtin_popcountll(hb);
                carry_lt += wave_read(i_lt, 63);
                carry_eq += wave_read(i_eq, 63);
            }
            // ---- the selection out of those slices' candidates: lane = candidate (token order inside a slice) ------
            constexpr int kAhead = 16;   // slices of the list whose candidates are in flight
            int cs[kAhead];
            float cp[kAhead];
            auto fetch = [&](int e, int& sel, float& phat) {
                const bool on = e < nlist;
                const size_t at = (hq * S + (on ? list_s[wave][e] : 0)) * AKV_MAX_TOPK + lane;
                sel = on ? a.cand_sel[at] : -1;
                phat = on ? a.cand_phat[at] : 0.0f;
            };
#pragma unroll
            for (int k = 0; k < kAhead; ++k) fetch(k, cs[k], cp[k]);
            for (int e = 0; e < nlist; e += kAhead) {
#pragma unroll
                for (int k = 0; k < kAhead; ++k) {
                    if (e + k < nlist) {   // uniform
                        const int jj = cs[k] >> 24, t = cs[k] & 0xFFFFFF;
                        const bool is_lt = cs[k] >= 0 && jj < J, is_eq = cs[k] >= 0 && jj == J;
                        const uint64_t b_lt = __ballot(is_lt), b_eq = __ballot(is_eq);
                        const int n_lt = list_lt[wave][e + k] + __builtin_amdgcn_mbcnt_hi((uint32_t)(b_lt >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)b_lt, 0));
                        const int n_eq = list_eq[wave][e + k] + __builtin_amdgcn_mbcnt_hi((uint32_t)(b_eq >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)b_eq, 0));
                        if (is_lt || (is_eq && n_eq < fromcut)) {
                            const int pos = n_lt + (n_eq < fromcut ? n_eq : fromcut);
                            ms.sel[wave][pos] = t;
                            ms.phat[wave][pos] = cp[k];
                        }
                    }
                    fetch(e + k + kAhead, cs[k], cp[k]);
                }
            }
        }
        __syncthreads();
        // all threads: the selected V rows of every head of this round are asked for, then used head by head
        OestRows<NT> rows[kWaves < G ? kWaves : G];
#pragma unroll
        for (int w = 0; w < (kWaves < G ? kWaves : G); ++w)
            if (g0 + w < G) mid_oest_fetch<NT>(a, bh, kk, ms, w, rows[w]);
#pragma unroll
        for (int w = 0; w < (kWaves < G ? kWaves : G); ++w)
            if (g0 + w < G) mid_oest_finish<NT>(a, size_t(b) * Hq + size_t(h) * G + g0 + w, kk, ms, w, rows[w], ehat);   // ends with a barrier
    }
    if (tid < kD) {
        a.Ehat[bh * kD + tid] = ehat;
        if (a.dbg.Ehat) a.dbg.Ehat[bh * kD + tid] = (int16_t)ehat;
    }
}

// Workgroup = kVWaves waves, one (sequence, KV head, kVChunk-token chunk); wave w takes the batches of rows
// w, w + kVWaves, ... of the chunk.  Groups of four or eight query heads run v_rows in its shared mode: every wave
// fetches and assembles its rows once, the rows pass through LDS, and the sums over rows for all heads of the group
// are matrix products on the matrix cores.
template <int G> constexpr bool v_shared() { return G >= kVWaves; }
template <int G, bool DEBUG>
__global__ __launch_bounds__(64 * kVWaves) void split_v_kernel(DecodeArgs a)
{
    constexpr bool SHARED = v_shared<G>();
    constexpr int KG = G >= 8 ? 1 : 2, RB = 8 * KG;         // one lane per (row of the batch, query head): at most 64 / G rows
    struct Private { float red[kVWaves][G][kD]; };
    struct Shared { union { VShare<G, RB> rows; float red[G][kD]; }; };   // the sums are laid down when the last round has been read
    __shared__ std::conditional_t<SHARED, Shared, Private> lds_s;
    __shared__ float z_s[kVWaves][G];
    __shared__ int last_s;

    const int h = blockIdx.y, b = blockIdx.z, split = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = lane >> 3, cl = lane & 7;
    const int Hkv = a.s.Hkv, Hq = a.s.Hq, Ncap = a.s.Ncap;
    const int len = min(min(a.lens[b], Ncap), a.max_len);   // a hint below the true length: the tokens past it are left out, consistently in all four kernels
    const int vchunk = a.vchunk;   // tokens per workgroup: a multiple of kVChunk chosen at launch
    const int c0 = split * vchunk;
    const size_t bh = size_t(b) * Hkv + h;
    const int nsplit = v_splits(Ncap);
    if (c0 >= len) {                                    // uniform: chunk beyond the sequence
        if (len == 0 && split == 0)                     // an empty sequence attends to nothing: zeros
            for (int idx = tid; idx < G * kD; idx += 64 * kVWaves)
                store_out(a, size_t(b) * Hq + size_t(h) * G + idx / kD, idx % kD, 0.0f);
        return;
    }

    VRule vr;
    v_rule_setup(a.Ehat + bh * kD, a.guard_bits, a.force_level, vr);
    float Mg[G];
#pragma unroll
    for (int g = 0; g < G; ++g) Mg[g] = a.M[size_t(b) * Hq + size_t(h) * G + g];
    float acc[SHARED ? 1 : G][SHARED ? 8 : 16], z[G];
#pragma unroll
    for (int g = 0; g < G; ++g) z[g] = 0.0f;
#pragma unroll
    for (int g = 0; g < (SHARED ? 1 : G); ++g)
#pragma unroll
        for (int i = 0; i < (SHARED ? 8 : 16); ++i) acc[g][i] = 0.0f;
    // HI bytes fetched three or four batches ahead in the private mode (few waves per SIMD: each keeps more bytes in
    // flight), two in the shared mode (four waves per SIMD; three and four measured 1.5 % and 3 % slower)
    constexpr int DL = SHARED ? 2 : (G == 2 ? 4 : 3);
    const u32x4_t none[1][KG] = {};
    if constexpr (SHARED) {
        v_rows<G, KG, DEBUG, 0, DL, true, true>(a, b, h, c0 + wave * RB, RB * kVWaves, vchunk / (RB * kVWaves), len, vr, Mg, acc, z, none, false, nullptr, 0, &lds_s.rows);
#pragma unroll
        for (int g = 0; g < G; ++g)
            for (int o = 1; o < 64; o <<= 1) z[g] += __shfl_xor(z[g], o);
        // a result tile holds the high parts of the weights in its rows 0 .. G-1 and the low parts in rows G .. 2G-1:
        // lanes 16 * (G / 4) apart hold the two parts of one (query head, line)
        float part[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) part[i] = (acc[0][i] + __shfl(acc[0][i], (lane + 4 * G) & 63)) * (1.0f / kVWeightScale);
        __syncthreads();   // every wave is done with the rows of the last round: the same LDS now takes the sums
        if (lane < 4 * G) {
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int i = 0; i < 4; ++i) lds_s.red[4 * (lane >> 4) + i][line_channel(32 * wave + 16 * t + (lane & 15))] = part[4 * t + i];
        }
    } else {
        v_rows<G, KG, DEBUG, 0, DL, true>(a, b, h, c0 + wave * RB, RB * kVWaves, vchunk / (RB * kVWaves), len, vr, Mg, acc, z, none, false);
        v_reduce_rows<G>(acc, z);
        if (r == 0) {
#pragma unroll
            for (int g = 0; g < G; ++g)
#pragma unroll
                for (int i = 0; i < 16; ++i) lds_s.red[wave][g][cl * 16 + i] = acc[g][i];
        }
    }
    if (lane == 0) {
#pragma unroll
        for (int g = 0; g < G; ++g) z_s[wave][g] = z[g];
    }
    __syncthreads();
    for (int idx = tid; idx < G * (kD + 1); idx += 64 * kVWaves) {
        const int g = idx / (kD + 1), d = idx % (kD + 1);
        float s = 0.0f;
#pragma unroll
        for (int w = 0; w < kVWaves; ++w) {
            if (d == kD) s += z_s[w][g];
            else if constexpr (SHARED) s += w == 0 ? lds_s.red[g][d] : 0.0f;
            else s += lds_s.red[w][g][d];
        }
        const size_t hq = size_t(b) * Hq + size_t(h) * G + g;
        if (d < kD) store_agent(&a.partO[(hq * nsplit + split) * kD + d], s);
        else store_agent(&a.partZ[hq * nsplit + split], s);
    }

    // ---- the workgroup that finishes last for this (sequence, KV head) combines the chunks -------------
    // out = sum_chunks O / sum_chunks Z: every chunk used the same global max, so nothing is rescaled.
    const int used = (len + vchunk - 1) / vchunk;
    stores_done();
    __syncthreads();
    if (tid == 0) last_s = take_ticket(&a.vcount[bh]) == used - 1;
    __syncthreads();
    if (!last_s) return;
    for (int idx = tid; idx < G * kD; idx += 64 * kVWaves) {
        const int g = idx / kD, d = idx % kD;
        const size_t hq = size_t(b) * Hq + size_t(h) * G + g;
        float o = 0.0f, zsum = 0.0f;
        for (int sp0 = 0; sp0 < used; sp0 += 8) {   // eight chunks' words in flight; the additions stay in chunk order
            float po[8], pz[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const bool on = sp0 + i < used;
                po[i] = on ? load_agent(&a.partO[(hq * nsplit + sp0 + i) * kD + d]) : 0.0f;
                pz[i] = on ? load_agent(&a.partZ[hq * nsplit + sp0 + i]) : 0.0f;
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                o += po[i];
                zsum += pz[i];
            }
        }
        store_out(a, hq, d, o / zsum);
    }
    if (tid == 0) store_agent(&a.vcount[bh], 0);   // ready for the next call
}

// what the register and LDS budgets of split_v_kernel<G> leave room for
int split_v_workgroups_per_cu(int G)
{
    if (G >= kVWaves) return 4;   // shared mode: 104 registers, 39 KB of LDS
    return G <= 1 ? 4 : (G <= 2 ? 3 : (G <= 4 ? 2 : 1));
}

template <int G>
static hipError_t launch_split_g(const DecodeArgs& a, hipStream_t st, hipEvent_t k_done_event, hipEvent_t mid_event)
{
    const int tile = kTB * kKWaves;   // tokens per workgroup of the K kernel: one 256-token block per wave
    const dim3 kgrid((a.max_len + tile - 1) / tile, a.s.Hkv, a.s.B), kblock(64 * kKWaves);
    hipLaunchKernelGGL((split_k_kernel<G>), kgrid, kblock, 0, st, a);
    if (hipError_t e = hipGetLastError()) return e;
    if (k_done_event)
        if (hipError_t e = hipEventRecord(k_done_event, st)) return e;
    hipLaunchKernelGGL((split_slice_kernel<G>), kgrid, dim3(256), 0, st, a);   // one workgroup per slice here as well
    if (hipError_t e = hipGetLastError()) return e;
    hipLaunchKernelGGL((split_select_kernel<G>), dim3(a.s.Hkv, a.s.B), dim3(256), 0, st, a);
    if (hipError_t e = hipGetLastError()) return e;
    if (mid_event)
        if (hipError_t e = hipEventRecord(mid_event, st)) return e;
    const dim3 vgrid((a.max_len + a.vchunk - 1) / a.vchunk, a.s.Hkv, a.s.B), vblock(64 * kVWaves);
    if (a.dbg.needV || a.dbg.appliedV || a.stats) hipLaunchKernelGGL((split_v_kernel<G, true>), vgrid, vblock, 0, st, a);
    else hipLaunchKernelGGL((split_v_kernel<G, false>), vgrid, vblock, 0, st, a);
    return hipGetLastError();
}

hipError_t launch_decode_split(const DecodeArgs& a, hipStream_t st, hipEvent_t k_done_event, hipEvent_t mid_event)
{
    switch (a.s.Hq / a.s.Hkv) {
        case 1: return launch_split_g<1>(a, st, k_done_event, mid_event);
        case 2: return launch_split_g<2>(a, st, k_done_event, mid_event);
        case 4: return launch_split_g<4>(a, st, k_done_event, mid_event);
        case 8: return launch_split_g<8>(a, st, k_done_event, mid_event);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace akv
