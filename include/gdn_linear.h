/*
 * gdn_linear — the projections of the layers around the resumed recurrence, for one MI355X
 * (gfx950).  Same library and conventions as gdn_resume.h (device pointers owned by the caller,
 * validation before anything is enqueued, negative error codes, no allocation, no stream
 * synchronisation).
 *
 * Why it belongs to the path: the paper times a layer group of one full-attention and three
 * GatedDeltaNet layers (Sec. 6, prototype wall-clock time); in such a layer the input and output
 * projections are the largest dense products a replayed suffix token pays for.  The paper does not
 * restate them; what is computed is the affine map of any such layer,
 *
 *     y[t][n] = bias[n] + sum_k x[t][k] w[n][k] ,      t < T, n < N, k < K,
 *
 * with the weight stored [out][in] (row n of w makes output n).
 *
 *   x      device, bf16, T rows of K elements at ldx elements (ldx >= K)
 *   w      device, bf16, N rows of K elements at ldw elements (ldw >= K)
 *   bias   device, fp32, N elements, or NULL
 *   y      device, out_dtype (GDN_BF16 or GDN_F32), T rows of N elements at ldy elements (ldy >= N):
 *          y may be a column slice of a wider buffer
 *   K a multiple of 64; x, w 16-byte aligned with ldx, ldw multiples of 8; y 8-byte aligned (bf16)
 *   or 16-byte aligned (fp32) with ldy a multiple of 4.  T = 0 or N = 0 is legal and does nothing.
 * Arithmetic: bf16 products on the matrix cores, fp32 accumulation over k in the order of the
 * k index by blocks of 16; the bias is added in fp32; one rounding to out_dtype.
 * Errors: GDN_ERR_NULL, GDN_ERR_ALIGN, GDN_ERR_SHAPE (K not a multiple of 64, a leading dimension
 * smaller than its row, an unknown out_dtype), GDN_ERR_COUNT (a negative size, or a leading dimension of 4 Mi
 * elements and more: a 256-row tile is addressed with 31-bit byte offsets).
 */
#ifndef GDN_LINEAR_H
#define GDN_LINEAR_H

#include <stdint.h>

#include "gdn_resume.h"

#ifdef __cplusplus
extern "C" {
#endif

int32_t gdn_linear(const void *x, int64_t ldx, const void *w, int64_t ldw, const float *bias,
                   void *y, int64_t ldy, int32_t out_dtype,
                   int64_t T, int32_t N, int32_t K, void *stream);

/*
 * The same map with its outputs split by column range over several destinations, one launch: segment s holds
 * outputs seg_cols[s] .. seg_cols[s + 1] - 1 and goes to seg_y[s] (T rows of that many elements at seg_ld[s]
 * elements).  This is the in-projection of a GatedDeltaNet layer as the layer's front end wants it: one weight
 * matrix [conv input | z | a | b], four separate tensors (include/gdn_layer.h); N = seg_cols[n_seg].
 *   n_seg      1 .. 8
 *   seg_cols   host, n_seg + 1, seg_cols[0] = 0, strictly increasing; inner boundaries multiples of 8
 *   seg_y      host array of n_seg device pointers (alignment as y above);  seg_ld: host, n_seg, multiples of 4
 * Everything else as gdn_linear.  Errors as gdn_linear, and GDN_ERR_COUNT for n_seg outside 1 .. 8,
 * GDN_ERR_SHAPE for seg_cols not starting at 0 or not increasing or a seg_ld below its segment's width,
 * GDN_ERR_ALIGN for an inner boundary that is no multiple of 8.
 */
int32_t gdn_linear_split(const void *x, int64_t ldx, const void *w, int64_t ldw, const float *bias,
                         int32_t n_seg, const int32_t *seg_cols, void *const *seg_y, const int64_t *seg_ld,
                         int32_t out_dtype, int64_t T, int32_t K, void *stream);

/*
 * Tuning knob, not a method step: fixes the workgroup tile gdn_linear uses (0: 128 x 128; 1: 256 x 256 with four
 * waves; 2: 256 x 256 with eight waves; 3: 64 x 64, which needs K a multiple of 128 and gives way to 0 otherwise;
 * anything else: chosen per call from T, N and K, the default).  Every shape computes the same
 * sums in the same order, so the results do not depend on it.  Process-wide; returns the previous setting (-1 = per
 * call).
 */
int32_t gdn_linear_tune(int32_t shape);

#ifdef __cplusplus
}
#endif
#endif /* GDN_LINEAR_H */
