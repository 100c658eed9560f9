/*
 * akw.h -- C ABI of the precision-aligned weight GEMV for MI355X (gfx950); part of the same library as akv.h.
 *
 * What it computes (paper: arxiv 2409.16546): the precision-alignment framework applied to a weight
 * matrix, y = x W with W as the quantised operand (section "Precision Alignment in Uncertainty
 * Calculation": A W = A (W_quant +- dW); section "A Framework for Aligning Precision": the framework
 * proposes a precision for every parameter of the weights as well as of the KV cache, and an addend's
 * bit width is the bit width of the weight it comes from).  The result is not known before the product,
 * so the addends x_k * W[k][n] are aligned with each other (Rule 1), exactly as for the K cache:
 *   - W keeps every fp16 bit, re-arranged into three planes (first 8 / next 4 / last 4 bits; section
 *     "Dynamic Quantization"), row-major in the input feature k, plus rowmax[k] = max_n |W[k][n]|;
 *   - for the activation row x the magnitude of the addends of input feature k is bounded by
 *     |x_k| * rowmax[k]; the addend of the largest magnitude fixes the last place that matters, and
 *     row k of W is read at the first 8, the first 12 or all 16 bits, whichever is the fewest that
 *     reach that place (+ guard_bits); bits that are not read count as 100...;
 *   - y[b][n] = sum_k x[b][k] * W~[k][n], accumulated in binary32.
 * With several activation rows (B > 1) a row of W is read once, at the largest of their needs.
 *
 * Conventions: those of akv.h (device pointers owned by the caller unless named "host", nothing is
 * allocated or synchronised, work is enqueued on the caller's stream, akv_status / akv_last_error()).
 * Shapes: K % 8 == 0, K <= 2^20, N % 16 == 0, K * N < 2^31, 1 <= B <= AKW_MAX_B.
 * Every device array (planes, rowmax, W, x, y) is 16-byte aligned; a misaligned one is refused with AKV_EINVAL.
 */
#ifndef AKW_H
#define AKW_H

#include "akv.h"

#ifdef __cplusplus
extern "C" {
#endif

#define AKW_MAX_B 4 /* activation rows per call: a matrix-vector path; larger batches are a dense contraction */

/*
 * One weight matrix in planes (all device memory):
 *   hi  [K][N]    uint8  first 8 bits of W[k][n]
 *   mid [K][N/2]  uint8  next 4 bits; column 2i in the low nibble of byte i, 2i+1 in the high nibble
 *   lo  [K][N/2]  uint8  last 4 bits, same packing
 *   rowmax [K]    uint16 max over n of the magnitude bits (h & 0x7fff) of row k
 */
typedef struct akw_weights {
    int32_t K, N;
    uint8_t *hi, *mid, *lo;
    uint16_t *rowmax;
} akw_weights;

typedef struct akw_sizes {
    size_t hi, mid, lo; /* planes                                              */
    size_t rowmax;      /* uint16 [K]                                          */
    size_t workspace;   /* scratch of akw_gemv for B <= AKW_MAX_B (256-B aligned) */
} akw_sizes;

/* Byte sizes of the caller-owned buffers of a K x N matrix (host call). */
akv_status akw_layout_sizes(int32_t K, int32_t N, akw_sizes *out);

/* Zero the counters in the workspace, once after allocating it (the kernels leave them at zero). */
akv_status akw_workspace_init(int32_t K, int32_t N, void *workspace, size_t workspace_bytes, void *stream);

/*
 * W: fp16 bit patterns [K][N], row-major -> the planes and rowmax of w ("Dynamic Quantization": all 16
 * bits are kept, so that any precision can be read later).  Lossless: akw_unpack returns W bit for bit.
 */
akv_status akw_pack(const akw_weights *w, const uint16_t *W, void *stream);
akv_status akw_unpack(const akw_weights *w, uint16_t *W_out, void *stream);

typedef struct akw_params {
    int32_t guard_bits;  /* 0..12: extra mantissa bits the rule keeps                                */
    int32_t force_level; /* -1: Rule 1; 0 / 1 / 2: read every row at 8 / 12 / 16 bits (2 = control)  */
    uint8_t *lvl_out;    /* NULL, or device uint8 [K]: the level each row of W was read at (export)  */
} akw_params;

/*
 * y[b][n] = sum_k x[b][k] * W~[k][n] for b < B.  x: fp16 bit patterns [B][K]; y: float [B][N].
 * params may be NULL (guard 0, Rule 1, no export).  workspace: akw_sizes.workspace bytes, 256-B aligned,
 * initialised once with akw_workspace_init; calls that share a workspace must not overlap in time.
 * Errors: AKV_EINVAL (shape, NULL pointer, parameter out of range), AKV_EWORKSPACE, AKV_EHIP.
 */
akv_status akw_gemv(const akw_weights *w, const uint16_t *x, int32_t B, float *y, const akw_params *params,
                    void *workspace, size_t workspace_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* AKW_H */
