/*
 * akv.h -- C ABI of the AlignedKV decode-attention library for MI355X (gfx950).
 *
 * What the library computes (paper: arxiv 2409.16546, "AlignedKV"):
 *   - a KV cache that keeps every fp16 bit of K and V, re-arranged so that the
 *     first 8 bits, the next 4 bits and the last 4 bits of every element lie in
 *     separately contiguous planes (section "Dynamic Quantization", the data
 *     re-arrangement figure), plus K_colmax, the per-column maximum of |K|
 *     (section "Quantization of K-Cache");
 *   - decode attention for ONE query token per sequence,
 *     S = QK^T/sqrt(D); S = softmax(S); O = SV  (section "Runtime of AlignedKV"),
 *     reading each K column at the precision Rule 1 (addend alignment) assigns
 *     it from q and K_colmax, and each V token row at the precision Rule 2
 *     (result alignment) assigns it from the scores and an approximate-top-k
 *     estimate O_est of the result (sections "A Framework for Aligning
 *     Precision", "Quantization of K-Cache", "Quantization of V-Cache");
 *     bits that are not read are filled with 100...
 *
 * Conventions
 *   - Every pointer in akv_cache, and q / out / k_new / v_new / workspace, is a
 *     DEVICE pointer owned by the caller; the library never allocates, frees or
 *     keeps device memory and never synchronises the device.  Pointers named
 *     "host" below are host pointers.
 *   - All device work is enqueued on the caller's stream (a hipStream_t passed
 *     as void*; NULL = the default stream) and is asynchronous.
 *   - Every function returns an akv_status; on error nothing was enqueued and
 *     akv_last_error() (host, thread-local) describes the reason.
 *   - fp16 data are IEEE binary16 bit patterns (uint16_t).  Inputs must be
 *     finite; with Inf/NaN the cache bytes are still exact, masks and outputs
 *     are unspecified.
 *   - D must be 128 (the only head size of the paper's model), Hq % Hkv == 0,
 *     Hq/Hkv <= 8, Ncap % 256 == 0.
 */
#ifndef AKV_H
#define AKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum akv_status {
    AKV_OK = 0,
    AKV_EINVAL = 1,     /* bad shape, NULL pointer, parameter out of range   */
    AKV_EWORKSPACE = 2, /* workspace too small or misaligned (256 B)          */
    AKV_EHIP = 3,       /* a HIP launch failed; akv_last_error() has the text */
    AKV_ECAPACITY = 4   /* akv_check_capacity_sync: an append of that many tokens would not fit */
} akv_status;

/* Problem shape.  Hq query heads share Hkv KV heads in groups of G = Hq/Hkv
 * consecutive query heads (query head hq uses KV head hq / G). */
typedef struct akv_shape {
    int32_t B;    /* sequences                      */
    int32_t Hq;   /* query heads                    */
    int32_t Hkv;  /* KV heads                       */
    int32_t D;    /* head dimension, must be 128    */
    int32_t Ncap; /* token capacity, multiple of 256 */
} akv_shape;

/* Byte sizes of every caller-owned buffer for a shape. */
typedef struct akv_sizes {
    size_t k_hi, k_mid, k_lo; /* K planes                                              */
    size_t v_hi, v_mid, v_lo; /* V planes                                              */
    size_t colmax;            /* uint16 [B][Hkv][D]                                    */
    size_t lens;              /* int32  [B]                                            */
    size_t flags;             /* int32  [AKV_NFLAGS + B]                               */
    size_t workspace;         /* scratch of akv_decode_attention (256-B aligned)       */
    size_t fp16_workspace;    /* scratch of akv_fp16_decode_attention (256-B aligned)  */
} akv_sizes;

#define AKV_TB 256          /* tokens per K block */
#define AKV_NFLAGS 4
#define AKV_FLAG_OVERFLOW 0 /* flags[0]: number of (call, sequence) appends refused for capacity */
#define AKV_FLAG_MAXLEN 1   /* flags[1]: number of (decode call, sequence) pairs whose length exceeded params->max_len
                               (the tokens past max_len were then left out of that call's attention)            */

/*
 * The cache: plane layout (TB = 256, NB = Ncap/256, all uint8 unless said):
 *   k_hi  [B][Hkv][NB][D][256]   first 8 bits of K, channel-major inside a block
 *   k_mid [B][Hkv][NB][D][128]   next 4 bits; token 2i in the low nibble of byte i, 2i+1 in the high nibble
 *   k_lo  [B][Hkv][NB][D][128]   last 4 bits, same packing
 *   v_hi  [B][Hkv][Ncap][D]      first 8 bits of V, token-major
 *   v_mid [B][Hkv][Ncap][D/2]    next 4 bits; channel 2i low nibble, 2i+1 high nibble
 *   v_lo  [B][Hkv][Ncap][D/2]    last 4 bits, same packing
 *   colmax[B][Hkv][D] uint16     max over stored tokens of (k & 0x7fff)   (K_colmax)
 *   lens  [B] int32              tokens stored per sequence
 *   flags [AKV_NFLAGS + B] int32 sticky device-side status words, then one arrival counter per sequence
 *                                used inside akv_append (zero between calls)
 * Slots that were never written hold zero after akv_cache_reset.
 * Alignment: the planes and colmax 16 bytes, lens and flags 4 bytes; every other device array an entry point takes
 * (q, out, k_new, v_new, k, v, k_out, v_out) 16 bytes.  A misaligned pointer is refused with AKV_EINVAL.
 */
typedef struct akv_cache {
    akv_shape shape;
    uint8_t *k_hi, *k_mid, *k_lo;
    uint8_t *v_hi, *v_mid, *v_lo;
    uint16_t *colmax;
    int32_t *lens;
    int32_t *flags;
} akv_cache;

/* Optional exports of the decisions (all device pointers, each may be NULL).
 * Entries for tokens t >= lens[b] are not written. */
typedef struct akv_debug {
    uint8_t *lvlK;     /* [B][Hkv][D]        level (0/1/2 = 8/12/16 bits) each K column was read at   */
    float *logits;     /* [B][Hq][Ncap]      q . K~, fp32, channels accumulated in ascending order    */
    int8_t *a;         /* [B][Hq][Ncap]      floor(log2(unnormalised softmax weight)), floored at -64 */
    int32_t *sel;      /* [B][Hq][topk]      tokens chosen by the approximate top-k, ascending, -1 padded */
    float *oest;       /* [B][Hq][D]         O_est                                                    */
    int16_t *Ehat;     /* [B][Hkv][D]        result exponent used by Rule 2 (min over the head group) */
    uint8_t *needV;    /* [B][Hkv][Ncap][D]  level each V element needs                               */
    uint8_t *appliedV; /* [B][Hkv][Ncap]     level each V token row was read at (max over its channels) */
} akv_debug;

/*
 * Optional device counters of what a decode call read (section "Reduction in Bit Widths": the average number of
 * bits fetched per element is the quantity the paper plots against the context length).  A DEVICE pointer to this
 * struct goes into akv_params.stats; the call ADDS to the counters (the caller zeroes them when it wants a fresh
 * count), inside the decode kernels themselves -- no further pass over the cache.  Index = level 0 / 1 / 2 =
 * 8 / 12 / 16 bits.  Only tokens t < lens[b] count.
 *   k_elems[l]      K elements read at level l              (columns at level l  x  tokens of the sequence)
 *   v_row_elems[l]  V elements read at level l              (token rows fetched at level l  x  D)
 *   v_need_elems[l] V elements that need level l by Rule 2  (before the maximum over the token row is taken)
 * Bytes fetched per plane follow: K_hi = sum_l k_elems[l], K_mid = (k_elems[1] + k_elems[2]) / 2, K_lo =
 * k_elems[2] / 2, and the same for V from v_row_elems.  Requesting the counters selects the kernel variant that also
 * serves the mask exports of akv_debug (slower than the plain one; results are identical).
 */
typedef struct akv_stats {
    uint64_t k_elems[3];
    uint64_t v_row_elems[3];
    uint64_t v_need_elems[3];
} akv_stats;

typedef struct akv_params {
    float scale;          /* softmax scale; <= 0 means 1/sqrt(D)                                    */
    int32_t topk;         /* size of the approximate top-k behind O_est, 1..AKV_MAX_TOPK; 0 means 32 */
    int32_t guard_bits;   /* extra mantissa bits both rules require, 0..12 (0 = the literal rule)    */
    int32_t force_level;  /* -1 adaptive; 0/1/2 read everything at 8/12/16 bits (2 = control group)  */
    int32_t out_dtype;    /* 0: out is float32 [B][Hq][D]; 1: out is fp16 [B][Hq][D]                 */
    int32_t max_len;      /* host-known upper bound of lens[] used to size the launch; 0 means Ncap.  In
                             akv_append_decode_attention it bounds the lengths AFTER the append.  A sequence
                             longer than max_len is attended over its first max_len tokens only (on either
                             path) and counted in flags[AKV_FLAG_MAXLEN]                               */
    const akv_debug *dbg; /* host pointer to a struct of device pointers, or NULL                    */
    void *const *events;  /* host pointer to AKV_NEVENTS hipEvent_t, or NULL: the library records them on the
                             stream so that a caller can time the kernels in place -- [0] before its first
                             kernel, [1] in front of the K kernel (after the append kernel where
                             akv_append_decode_attention runs one), [2] after the K kernel, [3] in front of
                             the V kernel, [4] after its last kernel.  On the head-per-workgroup path, which
                             is one kernel, [1], [2] and [3] follow [0] at once                        */
    int32_t path;         /* 0: choose; 1: head-per-workgroup path (one kernel; needs Hq/Hkv <= 4);
                             2: token-split path (four kernels).  Both give the same decisions.       */
    akv_stats *stats;     /* DEVICE pointer to counters the call adds to, or NULL                    */
} akv_params;

#define AKV_MAX_TOPK 64
#define AKV_NEVENTS 5

/* Library version (major*100 + minor). */
int akv_version(void);

/* Text of the last error on this host thread ("" if none). */
const char *akv_last_error(void);

/* Sizes of all buffers for a shape (host computation only).  AKV_EINVAL if the
 * shape breaks the conventions above. */
akv_status akv_layout_sizes(const akv_shape *shape, akv_sizes *out);

/* Zero lens, colmax, flags and every plane ("Dynamic Quantization": the cache
 * starts empty).  cache: host pointer to a struct of device pointers. */
akv_status akv_cache_reset(const akv_cache *cache, void *stream);

/*
 * Append tokens ("Dynamic Quantization": data are stored as fp16 and only
 * quantised when used; "Quantization of K-Cache": K_colmax is maintained while
 * storing).  k_new, v_new: device fp16 [B][Hkv][n][D].  n_new: device int32 [B]
 * with the number of leading rows (0..n) to take for each sequence, or NULL for
 * all n.  Tokens go to positions lens[b] .. lens[b]+n_new[b]-1; lens and colmax
 * are updated.  A sequence whose new length would exceed Ncap is left unchanged
 * and flags[AKV_FLAG_OVERFLOW] is incremented.  Calls on one cache must be
 * ordered on one stream.
 */
akv_status akv_append(const akv_cache *cache, const uint16_t *k_new, const uint16_t *v_new, const int32_t *n_new,
                      int32_t n, void *stream);

/*
 * Debugging aid, the one call that synchronises: waits for the work enqueued on `stream`, copies lens to the host and
 * returns AKV_ECAPACITY (naming the first sequence in akv_last_error()) if an append of n tokens to every sequence
 * would exceed Ncap for any of them, AKV_OK otherwise.  The appending calls themselves never synchronise: on the device
 * a sequence that would overflow is left unchanged and counted in flags[AKV_FLAG_OVERFLOW] ("Dynamic Quantization":
 * tokens are stored as they are produced; capacity is the caller's to provide).
 */
akv_status akv_check_capacity_sync(const akv_cache *cache, int32_t n, void *stream);

/*
 * Prepare a decode workspace: zero its control words (arrival counters that the
 * kernels of akv_decode_attention leave at zero again on exit).  Call it once on
 * every workspace before its first use, and again if anything else wrote to it.
 * For callers that cannot know: it is a single small fill kernel on the stream.
 */
akv_status akv_workspace_init(const akv_shape *shape, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Decode attention for one query token per sequence over the cache (sections
 * "Quantization of K-Cache", "Quantization of V-Cache", "Runtime of
 * AlignedKV").  q: device fp16 [B][Hq][D].  out: device [B][Hq][D] of
 * params->out_dtype.  A sequence with lens[b] == 0 yields zeros.  workspace:
 * device scratch of at least akv_sizes.workspace bytes, 256-B aligned, prepared
 * by akv_workspace_init; apart from its control words its contents are undefined
 * afterwards; concurrent calls need distinct workspaces.
 * params may be NULL (defaults: adaptive, topk 32, guard 0, float32 out).
 */
akv_status akv_decode_attention(const akv_cache *cache, const uint16_t *q, void *out, const akv_params *params,
                                void *workspace, size_t workspace_bytes, void *stream);

/* Which kernels akv_decode_attention takes for this shape when params->path is 0: 1 = head-per-workgroup (one
 * kernel, logits through the workspace), 3 = the same with the logits kept in LDS (none written to memory),
 * 2 = token-split (four kernels); max_len as in akv_params (0 means Ncap).  Host computation; 0 on a bad shape.
 * For callers that attribute time and bytes to kernels. */
int32_t akv_decode_path(const akv_shape *shape, int32_t max_len);

/*
 * akv_decode_attention for callers that cannot allocate device memory or keep a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid allocation.  Same arguments and results as
 * akv_decode_attention, but the scratch memory is a file-scope device array of AKV_STATIC_SCRATCH_BYTES inside the
 * library (one copy per GPU, held until the process ends); the call allocates and frees nothing.  A shape whose
 * workspace (akv_sizes.workspace + 64 KiB) exceeds that size, or with B * Hkv > 8192, is refused with
 * AKV_EWORKSPACE and a text that names both sizes.  Every call on a GPU shares that GPU's array: calls that
 * overlap on one GPU (two streams, two threads) race; order them on one stream.  The control words the kernels
 * rely on lie at a fixed place at the front of the array, are zeroed by a fill kernel on the first call on each
 * device and are left at zero by every call, so a call may follow one of any other shape.  The first call on a device
 * looks up the array's address (hipGetSymbolAddress): make that call before a stream capture begins; later calls
 * enqueue kernels only and can be captured into a HIP graph and replayed.
 */
#define AKV_STATIC_SCRATCH_BYTES (48u << 20)
akv_status akv_decode_attention_static(const akv_cache *cache, const uint16_t *q, void *out, const akv_params *params,
                                       void *stream);

/*
 * One decode step in one call: append one token per sequence (k_new, v_new:
 * device fp16 [B][Hkv][D], as akv_append with n = 1 and n_new = NULL), then
 * akv_decode_attention over the cache including that token.  Same results as
 * the two calls in a row; on the head-per-workgroup path both run in one
 * kernel.  A sequence that is already full keeps its tokens (the refusal is
 * counted in flags[AKV_FLAG_OVERFLOW]) and is attended as it is.
 */
akv_status akv_append_decode_attention(const akv_cache *cache, const uint16_t *k_new, const uint16_t *v_new,
                                       const uint16_t *q, void *out, const akv_params *params, void *workspace,
                                       size_t workspace_bytes, void *stream);

/* Lossless inverse of append: planes -> device fp16 k_out, v_out [B][Hkv][Ncap][D]
 * (all Ncap slots; unwritten slots give zero).  Either output may be NULL. */
akv_status akv_unpack(const akv_cache *cache, uint16_t *k_out, uint16_t *v_out, void *stream);

/*
 * The unquantised yardstick: the same decode attention on plain fp16 tensors
 * k, v: device [B][Hkv][Ncap][D] ("Runtime of AlignedKV", the 16-bit
 * baseline), lens: device int32 [B], q / out as above.  workspace: at least
 * akv_sizes.fp16_workspace bytes, 256-B aligned.
 */
akv_status akv_fp16_decode_attention(const akv_shape *shape, const uint16_t *k, const uint16_t *v, const int32_t *lens,
                                     const uint16_t *q, void *out, float scale, int32_t out_dtype, int32_t max_len,
                                     void *workspace, size_t workspace_bytes, void *stream);

/*
 * Measurement aid: read `bytes` bytes (16-byte aligned, a multiple of 16) of
 * device memory at buf once with a plain streaming kernel and discard them.
 * Timed by a caller, it gives the read ceiling of the device that the decode
 * kernels' effective bandwidth is put beside (decoding is bound by memory
 * access, the premise of the paper's introduction).  sink: device uint32,
 * never read, practically never written.  Nothing is allocated; asynchronous
 * on stream.
 */
akv_status akv_stream_read(const void *buf, size_t bytes, uint32_t *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* AKV_H */
