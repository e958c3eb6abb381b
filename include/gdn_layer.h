/*
 * gdn_layer — the elementwise front and back ends of a GatedDeltaNet layer around the resumed
 * recurrence of gdn_resume.h, for one MI355X (gfx950).  Same library, same conventions (host /
 * device pointers, validation before anything is enqueued, negative error codes, no
 * allocation, no stream synchronisation except the wait for an earlier call's plan upload).
 *
 * Why it belongs to the path: the paper's method applies to layers whose hidden state can be
 * taken out and put back without loss (Sec. 1), and it times a layer group with GatedDeltaNet
 * layers (Sec. 6, prototype wall-clock time).  Besides the matrix state S, such a layer carries the last K-1 inputs of
 * its short convolution; a resumed request is exact only if those rows are checkpointed and
 * restored with S.  The paper does not restate the layer; what is computed is the published
 * GatedDeltaNet layer (projections excluded: they are plain GEMMs):
 *
 *   short convolution  y_t[c] = SiLU(bias[c] + sum_{j<K} w[c][j] x_{t-(K-1)+j}[c]),  x_s = 0 for s <= 0
 *                      (depthwise, causal; tap K-1 multiplies the current token)
 *   its state at c     rows x_{c-K+2} .. x_c, oldest first: [K-1][C] in the input type
 *   q, k               per head x / sqrt(sum x^2 + qk_eps) after the convolution;  v = y
 *   beta               sigmoid(b_pre)
 *   gate a             exp(-exp(A_log[h]) softplus(a_pre + dt_bias[h]))
 *   output             y = o / sqrt(mean(o^2) + norm_eps) * weight * SiLU(z) per (token, value head)
 *
 * Stacked layers: with L > 1 every tensor below gains a leading layer index -- token tensors are
 * [L][T_alloc][...] planes (the layout gdn_resume_prefill reads q, k, v, beta, gate in and writes o
 * in), parameters are [L][...], a convolution-state slot is [L][K-1][C] -- and one launch handles all
 * layers; the request and emit index arrays are shared by the layers.
 *
 * Channels of the convolution input: C = 2 H_qk d_k + H_v d_v, ordered [q heads | k heads | v heads].
 * Positions are absolute and 1-based as in gdn_resume.h: request r owns packed rows
 * [cu_seqlens[r], cu_seqlens[r+1]) = tokens at positions start_pos[r]+1 ...
 */
#ifndef GDN_LAYER_H
#define GDN_LAYER_H

#include <stdint.h>

#include "gdn_resume.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gdn_layer_shape {
    int32_t H_qk;       /* query/key heads */
    int32_t H_v;        /* value heads */
    int32_t d_k;        /* 64 or 128 */
    int32_t d_v;        /* 64 or 128 */
    int32_t conv_k;     /* taps K of the short convolution, 2..4 */
    int32_t in_dtype;   /* GDN_F32 or GDN_BF16: x_qkv, a_pre, b_pre, z and the convolution states */
    int32_t out_dtype;  /* GDN_F32 or GDN_BF16: q, k, v, beta, gate (what gdn_resume_prefill reads) and y */
    int32_t o_dtype;    /* GDN_F32 or GDN_BF16: the recurrence output o read by gdn_layer_output */
    float qk_eps;       /* inside the root of the q/k normalisation */
    float norm_eps;     /* inside the root of the output normalisation */
    int32_t L;          /* stacked layers handled by one call (>= 1), independent problems with their own
                           inputs and parameters, as in gdn_shape */
    int64_t T_alloc;    /* tokens per layer plane of the token tensors (>= the call's T); 0 = exactly T */
} gdn_layer_shape;

/* Bytes of device workspace gdn_layer_inputs needs (its index arrays).  Negative on error. */
int64_t gdn_layer_workspace_bytes(int32_t n_req, int32_t n_emit);

/*
 * Front end of the layer for a packed batch of resumed requests, one launch:
 *   q, k, v     from x_qkv by the short convolution continued from each request's stored state,
 *               SiLU, and the per-head L2 normalisation of q and k;
 *   beta, gate  from b_pre, a_pre;
 *   the convolution state at every emit position, stored to conv_dst.
 * Arguments
 *   x_qkv       device, in_dtype, [T][C] row-major (T = cu_seqlens[n_req])
 *   conv_w      device, fp32, [C][K];  conv_b: device, fp32, [C], or NULL (no bias)
 *   a_pre,b_pre device, in_dtype, [T][H_v];  A_log, dt_bias: device, fp32, [H_v]
 *   cu_seqlens  host, n_req + 1;  start_pos: host, n_req (position of the loaded state)
 *   conv_src    device, in_dtype, slots of [K-1][C] at src_slot_stride elements; src_slot: host,
 *               n_req ids in [-1, n_src_slots), -1 = zeros (start of the sequence).  May be NULL
 *               when every id is -1.
 *   emit_cu, emit_pos, emit_slot   host, as in gdn_resume_prefill: positions strictly increasing
 *               per request in (start_pos[r], start_pos[r] + length]; ids in [0, n_dst_slots),
 *               all different.  conv_dst: device, in_dtype, slots at dst_slot_stride elements;
 *               may be NULL when there is no emission.
 *   q, k        device, out_dtype, [T][H_qk][d_k];  v: [T][H_v][d_v];  beta, gate: [T][H_v]
 *   workspace   device, 16-byte aligned, >= gdn_layer_workspace_bytes(n_req, n_emit)
 * Errors: GDN_ERR_NULL, _ALIGN (pointers and slot strides 16-byte aligned), _SHAPE (also a slot
 * smaller than L (K-1) C), _SEQLENS (also more tokens than T_alloc),
 * _START, _EMIT, _SLOT_RANGE, _SLOT_DUP, _SLOT_HAZARD (an emit slot overlaps, by address, any
 * request's source slot: the launch reads and writes concurrently), _WORKSPACE, _COUNT.
 * A request of length 0 is legal: its states at start_pos[r] cannot be asked for (the emit
 * interval is empty).
 */
int32_t gdn_layer_inputs(const gdn_layer_shape *shape,
                         const void *x_qkv, const float *conv_w, const float *conv_b,
                         const void *a_pre, const void *b_pre, const float *A_log, const float *dt_bias,
                         int32_t n_req, const int32_t *cu_seqlens, const int32_t *start_pos,
                         const void *conv_src, int64_t src_slot_stride, int32_t n_src_slots,
                         const int32_t *src_slot,
                         const int32_t *emit_cu, const int32_t *emit_pos,
                         void *conv_dst, int64_t dst_slot_stride, int32_t n_dst_slots,
                         const int32_t *emit_slot,
                         void *q, void *k, void *v, void *beta, void *gate,
                         void *workspace, int64_t workspace_bytes, void *stream);

/*
 * Back end of the layer: y[t][h][:] = o[t][h][:] / sqrt(mean(o[t][h][:]^2) + norm_eps) * weight[:] * SiLU(z[t][h][:]).
 *   o       device, o_dtype, [T][H_v][d_v] (the recurrence output of gdn_resume_prefill, one layer)
 *   z       device, in_dtype, [T][H_v][d_v];  weight: device, fp32, [d_v]
 *   y       device, out_dtype, [T][H_v][d_v]
 * With L > 1: o, z, y are [L][T_alloc][H_v][d_v], weight [L][d_v].
 * Errors: GDN_ERR_NULL, _ALIGN, _SHAPE, _COUNT, _SEQLENS (T beyond T_alloc).  T = 0 is legal.
 */
int32_t gdn_layer_output(const gdn_layer_shape *shape, const void *o, const void *z, const float *weight,
                         void *y, int64_t T, void *stream);

#ifdef __cplusplus
}
#endif

#endif /* GDN_LAYER_H */
