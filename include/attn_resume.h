/*
 * attn_resume — the attention layers' side of a cache hit, for one MI355X (gfx950).  Same
 * library and conventions as gdn_resume.h (host / device pointers named per argument, validation
 * before anything is enqueued, negative error codes, no allocation, no stream synchronisation
 * except the wait for an earlier call's plan upload to leave its pinned staging buffer).
 *
 * Why it belongs to the path: the paper's hybrid runs keep the full attention KV cache beside
 * the sparse recurrent checkpoints (Table 1, caption), count the load of the cached keys and values as
 * the third part of a hit's cost (Sec. 6, overhead decomposition), and time a layer group with
 * one full attention layer (Sec. 6, prototype wall-clock time).  The paper does not restate attention;
 * what is computed is causal softmax attention of the recomputed suffix over the restored prefix:
 *
 *   request r resumed at position c = start_pos[r] (keys / values 1..c already in its cache
 *   rows 0..c-1) with suffix tokens c+1 .. c+n:
 *     cache rows c .. c+n-1  <-  k_new, v_new of the suffix                      (append)
 *     o_t[h] = sum_{j=1..t} softmax_j(scale * q_t[h] . k_j[g]) v_j[g],   g = h / (H_q / H_kv)
 *     y_t[h] = o_t[h] * sigmoid(gate_t[h])    when an output gate is passed (gated attention)
 *
 * Precision: inputs are bf16; logits, the running maximum and the normaliser are fp32.  The key
 * cache is bf16; the VALUE cache is kept in fp16 (the append widens bf16 to fp16: exact for
 * magnitudes in [2^-14, 65504], rounded to a multiple of 2^-24 below, infinite above), so that
 * the weights can enter the second contraction rounded to fp16 (2^-12 relative) rather than to
 * bf16 (2^-9); the normaliser is the sum of the rounded weights, so that the weights actually
 * used sum to one as in the definition.
 *
 * Cache layout: a pool of sequence slots, slot s at k_cache + s * slot_stride (elements), each
 * [cap][H_kv][d] row-major: token-major, so that the restored prefix of a request is ONE
 * contiguous range per tensor.  k and v pools have the same geometry (both 16-bit elements); one
 * slot holds less than 2 GiB per tensor ((cap + 128) * H_kv * d * 2 bytes < 2^31).
 */
#ifndef ATTN_RESUME_H
#define ATTN_RESUME_H

#include <stdint.h>

#include "gdn_resume.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct attn_shape {
    int32_t H_q;      /* query heads */
    int32_t H_kv;     /* key/value heads; H_q a multiple of it */
    int32_t d;        /* head size: 64, 128 or 256 */
    int32_t o_dtype;  /* GDN_F32 or GDN_BF16: type of o (and of the gate, which is bf16 always) */
    float scale;      /* logit multiplier, usually 1/sqrt(d); finite and > 0 */
} attn_shape;

/* Bytes of device workspace attn_suffix_prefill needs: its index arrays and, for calls with too few
 * (request, head, 128-token) pieces to fill the chip, the partial results of split key walks (a
 * fixed region of 768 x 128 x (d + 2) floats).  Negative on error. */
int64_t attn_workspace_bytes(const attn_shape *shape, int32_t n_req, int64_t total_tokens);

/*
 * Restore the cached prefix of n_req requests from a HOST pool with the same slot layout
 * (Sec. 6, overhead decomposition, part iii): rows 0 .. prefix_len[r]-1 of host slot
 * host_slot[r] go to the same rows of device slot seq_slot[r], k and v, as asynchronous copies
 * on `stream` (pinned host memory lets them overlap; pageable memory works but blocks the
 * host).  Bit-exact.
 *   host_k, host_v   host, bf16 / fp16 as on the device, slots at host_slot_stride elements;
 *                    host_slot: host, n_req ids
 *   k_cache, v_cache device, bf16 / fp16, slots at slot_stride elements;  seq_slot: host, n_req ids, distinct
 *   prefix_len       host, n_req, each in [0, cap]
 * Errors: GDN_ERR_NULL, _ALIGN (strides multiples of 8 elements), _SHAPE, _COUNT, _SLOT_RANGE,
 * _SLOT_DUP, _START (a prefix longer than cap).
 */
int32_t attn_kv_restore(const attn_shape *shape, int32_t n_req, const int32_t *prefix_len,
                        const void *host_k, const void *host_v, int64_t host_slot_stride,
                        int32_t n_host_slots, const int32_t *host_slot,
                        void *k_cache, void *v_cache, int64_t slot_stride, int32_t n_slots,
                        int32_t cap, const int32_t *seq_slot, void *stream);

/*
 * The reverse of attn_kv_restore: rows 0 .. n_rows[r]-1 of device slot seq_slot[r] go to the same
 * rows of host slot host_slot[r] (how a finished request's keys and values reach the host pool);
 * host_slot ids distinct.  Same argument meaning and errors.
 */
int32_t attn_kv_spill(const attn_shape *shape, int32_t n_req, const int32_t *n_rows,
                      void *host_k, void *host_v, int64_t host_slot_stride,
                      int32_t n_host_slots, const int32_t *host_slot,
                      const void *k_cache, const void *v_cache, int64_t slot_stride, int32_t n_slots,
                      int32_t cap, const int32_t *seq_slot, void *stream);

/*
 * Suffix prefill of the attention layer for a packed batch of resumed requests: appends the
 * suffix's keys and values to each request's cache rows and computes the attention output of
 * every suffix token over positions 1 .. its own (two launches on `stream`; three when the call
 * is small enough for key walks of 1024 keys and more to be split over workgroups, after which a
 * merge pass writes o).  Results do not depend on the batch a request is packed with as long as
 * its walk is not split.  attn_tune_split(0) keeps every walk whole; attn_tune_pack(0) keeps one
 * query head per workgroup also where suffixes are short (otherwise the heads of a key/value group
 * then share a workgroup's rows; results are bitwise the same either way).
 *   q            device, bf16, [T][H_q][d] (T = cu_seqlens[n_req]);  k_new, v_new: [T][H_kv][d]
 *   out_gate     device, bf16, [T][H_q][d], or NULL (no gate)
 *   cu_seqlens   host, n_req + 1;  start_pos: host, n_req, the restored prefix length c >= 0
 *   k_cache, v_cache  device, bf16 / fp16, the pools; rows [0, c) of slot seq_slot[r] hold the prefix;
 *                rows [c, c+n) are written by this call; seq_slot: host, n_req ids in
 *                [0, n_slots), distinct;  c + n <= cap
 *   o            device, o_dtype, [T][H_q][d]
 *   workspace    device, 16-byte aligned, >= attn_workspace_bytes(shape, n_req, T)
 * Errors: GDN_ERR_NULL, _ALIGN, _SHAPE, _SEQLENS, _START (negative, or c + n > cap), _COUNT,
 * _SLOT_RANGE, _SLOT_DUP, _WORKSPACE.  A request of length 0 is legal and does nothing.
 */
int32_t attn_suffix_prefill(const attn_shape *shape, const void *q, const void *k_new,
                            const void *v_new, const void *out_gate,
                            int32_t n_req, const int32_t *cu_seqlens, const int32_t *start_pos,
                            void *k_cache, void *v_cache, int64_t slot_stride, int32_t n_slots,
                            int32_t cap, const int32_t *seq_slot,
                            void *o, void *workspace, int64_t workspace_bytes, void *stream);

/*
 * The work list attn_suffix_prefill makes for a call (host only, integers; exposed for tests and
 * for callers that want to see the launch shape).  A unit is one workgroup's walk for each head
 * block: rows = 128 / *heads_per_row_group suffix tokens starting at token unit_tile * that many
 * of request unit_req (with *heads_per_row_group query heads of a key/value group per token: 1,
 * or H_q / H_kv in calls with short suffixes), key tiles [unit_t0, unit_t1) of *key_tile_rows rows
 * each; unit_part is the workspace slot of a part of a split walk, or -1 for a whole walk.  Units
 * come in launch order, most key tiles first.  The five arrays hold `capacity` entries;
 * *n_units is set also when that is too few (GDN_ERR_COUNT).
 */
int32_t attn_plan(const attn_shape *shape, int32_t n_req, const int32_t *cu_seqlens,
                  const int32_t *start_pos, int32_t capacity,
                  int32_t *unit_req, int32_t *unit_tile, int32_t *unit_t0, int32_t *unit_t1,
                  int32_t *unit_part, int32_t *n_units, int32_t *heads_per_row_group,
                  int32_t *key_tile_rows);

/*
 * Tuning knobs (not steps of the method; for tests and experiments).  attn_tune_split(0) forbids
 * cutting long key walks into parts, attn_tune_pack(0) forbids packing the query heads of a
 * key/value group into one workgroup's rows; a non-zero argument restores the automatic choice.
 * Each returns its previous setting (1 = automatic).  Process-wide; read at every call.
 */
int32_t attn_tune_split(int32_t allow);
int32_t attn_tune_pack(int32_t allow);

#ifdef __cplusplus
}
#endif

#endif /* ATTN_RESUME_H */
