/*
 * gdn_resume — resume-from-checkpoint GatedDeltaNet prefill with sparse checkpoint emission,
 * for one MI355X (gfx950).  C ABI: plain pointers and sizes, no framework types.
 *
 * The operation (Sec. 3 and Remark 1 of the paper, "Sparse Prefix Caching for Hybrid and
 * Recurrent LLM Serving"): a cached prefix of length N keeps exact recurrent states at a
 * sparse set of checkpoint positions C = {c_1 < ... < c_M}.  A request that overlaps the
 * prefix up to depth t loads the state of the deepest checkpoint l(t;C) = max({0} u {c <= t}),
 * replays only the tokens after it, and may store the exact states it passes at further
 * checkpoint positions.  The state "at position c" is the state after consuming tokens 1..c;
 * position 0 is the zero state.
 *
 * The recurrent update replayed is the gated delta rule of a GatedDeltaNet layer, per value
 * head, with state S (d_v x d_k, fp32, row-major [d_v][d_k]):
 *     S~ = a_t S_{t-1};  u_t = b_t (v_t - S~ k_t);  S_t = S~ + u_t k_t^T;  o_t = scale * S_t q_t.
 *
 * Conventions common to every entry point
 *   - "host" pointers are read during the call and may be freed on return; "device" pointers
 *     are HIP device memory owned by the caller and must stay valid until the work enqueued
 *     on `stream` has finished.  `stream` is a hipStream_t passed as void* (NULL = default).
 *   - No entry point allocates or frees device memory and none synchronises the stream,
 *     except that a call which uploads index arrays may wait (on the host) for the upload of
 *     the call eight such calls back to leave its pinned staging buffer (the library owns a
 *     ring of eight).
 *   - Every argument is validated on the host before anything is enqueued; on error nothing
 *     is enqueued and a negative code is returned.  HIP failures return GDN_ERR_HIP - hipError.
 *   - The library is written for one GPU per process (kernel attributes and the device's size
 *     are looked up once, on the device that is current at the first call); calls may come from
 *     several host threads and streams.
 *   - A checkpoint slot holds the states of all layers and value heads of one position:
 *     [L][H_v][d_v][d_k] fp32, contiguous; a pool is slots at a fixed stride (in floats).
 */
#ifndef GDN_RESUME_H
#define GDN_RESUME_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    GDN_OK = 0,
    GDN_ERR_NULL = -1,        /* a required pointer is NULL */
    GDN_ERR_ALIGN = -2,       /* a device pointer or stride is not 16-byte aligned */
    GDN_ERR_SHAPE = -3,       /* unsupported head size / dtype, H_v not a multiple of H_qk, ... */
    GDN_ERR_SEQLENS = -4,     /* cu_seqlens not starting at 0, decreasing, or beyond T_alloc */
    GDN_ERR_SLOT_RANGE = -5,  /* a slot id outside its pool (sources may be -1) */
    GDN_ERR_SLOT_DUP = -6,    /* two states written to the same destination slot */
    GDN_ERR_SLOT_HAZARD = -7, /* a destination slot overlaps (by address) a source slot that is not the writer's own */
    GDN_ERR_EMIT = -8,        /* emit positions not strictly increasing inside (start, end] */
    GDN_ERR_WORKSPACE = -9,   /* workspace NULL, misaligned or too small */
    GDN_ERR_START = -10,      /* negative start position, or positions overflowing int32 */
    GDN_ERR_COUNT = -11,      /* a negative count */
    GDN_ERR_STATIC_LIMIT = -12, /* gdn_resume_prefill_static: the call's chunk plan exceeds the library's static array */
    GDN_ERR_HIP = -1000       /* GDN_ERR_HIP - (int)hipError_t */
};

enum { GDN_F32 = 0, GDN_BF16 = 1 };

/* Number of tokens one chunk of the kernels covers (kernel-internal granularity; positions
 * need not be aligned to it). */
#define GDN_CHUNK 64

typedef struct gdn_shape {
    int32_t L;         /* stacked recurrent layers, independent problems with their own inputs */
    int32_t H_qk;      /* query/key heads */
    int32_t H_v;       /* value heads, a multiple of H_qk; value head h uses q/k head h / (H_v/H_qk) */
    int32_t d_k;       /* 64 or 128 */
    int32_t d_v;       /* 64 or 128 */
    int32_t in_dtype;  /* GDN_F32 or GDN_BF16: type of q, k, v, beta, gate */
    int32_t o_dtype;   /* GDN_F32 or GDN_BF16: type of o */
    float scale;       /* o_t = scale * S_t q_t; 1.0 for the plain definition */
    int64_t T_alloc;   /* tokens per layer plane of the token tensors (>= total tokens) */
} gdn_shape;

/*
 * Sec. 3, l(t;C): index i of the deepest checkpoint pos[i] <= t, or -1 when there is none
 * (resume from the zero state at position 0).  pos: host, M strictly increasing positions.
 * Pure host function.  Returns GDN_ERR_NULL (-1 cannot be told apart, so M > 0 with a NULL
 * pos returns -1 as well: "no checkpoint").
 */
int32_t gdn_deepest_ckpt(const int32_t *pos, int32_t M, int32_t t);

/*
 * Host-only chunk planner (exposed for tests; gdn_resume_prefill runs the same code).
 * Splits every request's token range at its emit positions and then into pieces of at most
 * GDN_CHUNK tokens.  Outputs (host arrays of `capacity` entries, req_chunk_cu of n_req+1):
 *   chunk_tok0[c]  first packed token of chunk c      chunk_len[c]  1..GDN_CHUNK tokens
 *   chunk_emit[c]  flat index into emit_pos of the emission at the end of chunk c, or -1
 *   req_chunk_cu   request r owns chunks [req_chunk_cu[r], req_chunk_cu[r+1])
 * Returns the number of chunks, GDN_ERR_WORKSPACE when capacity is too small, or the
 * validation error of the index arrays (GDN_ERR_SEQLENS / _START / _EMIT / _NULL / _COUNT).
 */
int32_t gdn_plan_chunks(int32_t n_req, const int32_t *cu_seqlens, const int32_t *start_pos,
                        const int32_t *emit_cu, const int32_t *emit_pos,
                        int32_t *chunk_tok0, int32_t *chunk_len, int32_t *chunk_emit,
                        int32_t *req_chunk_cu, int32_t capacity);

/*
 * Upper bound, in bytes, of the workspace gdn_resume_prefill needs for a call with this
 * shape, n_req requests, total_tokens packed tokens and n_emit emissions.  Negative on error.
 * The per-chunk intermediates are produced and consumed slab by slab (a bounded number of
 * chunks of every request at a time), so beyond one slab the bound does not grow with the
 * sequence length: it holds the chunk plan, one carried state per (request, layer, head) and
 * one slab.
 */
int64_t gdn_workspace_bytes(const gdn_shape *shape, int32_t n_req, int64_t total_tokens,
                            int32_t n_emit);

/*
 * The smaller workspace that suffices when the call is served by the fused kernel (bf16 inputs,
 * d_k = d_v = 128 or 64: preparation and recurrence of a chain in one workgroup, see gdn_tune_fused):
 * the chunk plan only.  A call given at least this much but less than gdn_workspace_bytes runs
 * the fused kernel whatever the library's estimate says; for other shapes the value equals
 * gdn_workspace_bytes.  Negative on error.
 */
int64_t gdn_workspace_bytes_fused(const gdn_shape *shape, int32_t n_req, int64_t total_tokens,
                                  int32_t n_emit);

/*
 * Checkpoint load (Sec. 6, overhead decomposition, item (i): loading the stored checkpoint),
 * here from a pool in HBM:  dst[i] = pool[slot_ids[i]] for i < n, zeros when slot_ids[i] == -1.
 *   pool      device, fp32, n_slots slots at slot_stride floats
 *   slot_ids  host, n ids in [-1, n_slots)
 *   dst       device, n states at dst_stride floats;  state_elems floats are copied per state
 * state_elems and both strides must be multiples of 4, pointers 16-byte aligned,
 * strides >= state_elems.  Bit-exact copy.  dst must not overlap the pool.
 */
int32_t ckpt_gather(const float *pool, int64_t slot_stride, int32_t n_slots,
                    const int32_t *slot_ids, int32_t n,
                    float *dst, int64_t dst_stride, int64_t state_elems, void *stream);

/*
 * Checkpoint store: pool[slot_ids[i]] = src[i] for i < n.  Same argument rules as
 * ckpt_gather; ids in [0, n_slots); a repeated id is GDN_ERR_SLOT_DUP.  Bit-exact copy.
 */
int32_t ckpt_scatter(float *pool, int64_t slot_stride, int32_t n_slots,
                     const int32_t *slot_ids, int32_t n,
                     const float *src, int64_t src_stride, int64_t state_elems, void *stream);

/*
 * The resumed prefill (Sec. 3: replay of tokens l+1..t from the state at l; Remark 1: the
 * result equals a full replay; Sec. 5 "Capturing checkpoints": states at checkpoint positions
 * are captured, here inside the same pass).
 *
 * Token tensors (device) are packed over requests, token-major, one plane per layer:
 *   q, k        [L][T_alloc][H_qk][d_k]        v, o   [L][T_alloc][H_v][d_v]
 *   beta, gate  [L][T_alloc][H_v]              gate is a_t in (0,1], not its logarithm
 * Request r owns packed tokens [cu_seqlens[r], cu_seqlens[r+1]); they are the tokens at
 * absolute positions start_pos[r]+1 .. of its sequence.  A zero-length request is legal and
 * does nothing.  bf16 inputs must be finite and below 65504 in magnitude (they are widened
 * exactly to fp16 for the matrix cores), and the states must stay below it too: on the bf16
 * path the state and the per-chunk updates enter the matrix cores rounded to fp16.
 *
 *   cu_seqlens  host int32 [n_req+1], cu_seqlens[0] == 0, non-decreasing, last <= T_alloc
 *   start_pos   host int32 [n_req], >= 0: position l_r of the loaded state
 *   state_src   device fp32 pool read for start states (may be NULL when every src_slot is -1)
 *   src_slot    host int32 [n_req] in [-1, src_n_slots): slot of the start state, -1 = zeros
 *   emit_cu     host int32 [n_req+1]; request r stores emissions [emit_cu[r], emit_cu[r+1])
 *   emit_pos    host int32 [n_emit]: absolute positions, strictly increasing per request,
 *               inside (start_pos[r], start_pos[r] + len_r]
 *   state_dst   device fp32 pool written with the emitted states (may equal state_src)
 *   emit_slot   host int32 [n_emit] in [0, dst_n_slots), all distinct.  Source and destination
 *               slots are compared by address (the pools may be the same memory, also under
 *               different base pointers): a destination may be the writer's own source slot
 *               (the very same memory), any other overlap with a source slot read by this call
 *               is GDN_ERR_SLOT_HAZARD
 *   o           device, written for every packed token
 *   workspace   device, 256-byte aligned, at least gdn_workspace_bytes(...) bytes; contents
 *               are scratch, nothing is carried between calls
 * Outputs: o within the stated tolerance of the token-by-token definition, emitted states
 * likewise, slot indexing exact.  Calls that share a workspace must be ordered on one stream.
 */
int32_t gdn_resume_prefill(const gdn_shape *shape,
                           const void *q, const void *k, const void *v,
                           const void *beta, const void *gate,
                           int32_t n_req, const int32_t *cu_seqlens, const int32_t *start_pos,
                           const float *state_src, int64_t src_slot_stride, int32_t src_n_slots,
                           const int32_t *src_slot,
                           const int32_t *emit_cu, const int32_t *emit_pos,
                           float *state_dst, int64_t dst_slot_stride, int32_t dst_n_slots,
                           const int32_t *emit_slot,
                           void *o, void *workspace, int64_t workspace_bytes, void *stream);

/*
 * gdn_resume_prefill for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, outputs and errors as gdn_resume_prefill without the workspace.  The call's chunk
 * plan (a few int32 per 64-token chunk and per request) lives in a static device array inside
 * the library, gdn_static_plan_capacity() bytes per GPU (512 KiB, held until the process ends;
 * enough for about 43 000 chunks, i.e. 2.7 M tokens per layer), and is written there by the
 * arguments of small launches on `stream`: no hipMalloc, no hipFree, no pinned staging buffer,
 * no host-to-device copy.  The fused kernel serves the call (bf16 inputs, d_k = d_v = 128 or 64; other
 * shapes return GDN_ERR_SHAPE; gdn_tune_fused does not apply); a plan beyond the capacity returns
 * GDN_ERR_STATIC_LIMIT before anything is enqueued.  Every call on a GPU uses that GPU's one array:
 * calls must be ordered on one stream (or otherwise not overlap in time), two overlapping calls
 * race on the plan.  Nothing in the array needs clearing between calls: a call overwrites the
 * part it reads.  Outputs are bitwise those of gdn_resume_prefill when that runs the fused kernel.
 */
int32_t gdn_resume_prefill_static(const gdn_shape *shape,
                                  const void *q, const void *k, const void *v,
                                  const void *beta, const void *gate,
                                  int32_t n_req, const int32_t *cu_seqlens, const int32_t *start_pos,
                                  const float *state_src, int64_t src_slot_stride, int32_t src_n_slots,
                                  const int32_t *src_slot,
                                  const int32_t *emit_cu, const int32_t *emit_pos,
                                  float *state_dst, int64_t dst_slot_stride, int32_t dst_n_slots,
                                  const int32_t *emit_slot,
                                  void *o, void *stream);
int64_t gdn_static_plan_capacity(void);

/*
 * Host tier (Sec. 5, implementation details: the prototype keeps checkpoints in CPU RAM;
 * Sec. 6: loading the stored checkpoint is the first component of the overhead of a hit).
 * Checkpoint states may live in a pinned host pool (allocate it with hipHostMalloc or an
 * equivalent; pageable memory works but the copies then block the host) with the same slot
 * layout as the device pool.
 *
 * ckpt_fetch_host: dev_pool[dev_ids[i]] = host_pool[host_ids[i]], i < n, as asynchronous
 * copies on `stream`; dev_ids distinct.  ckpt_spill_host: the reverse; host_ids distinct.
 * Strides in floats, multiples of 4; ids inside their pools (no -1).  Bit-exact.
 *
 * gdn_resume_prefill_host: gdn_resume_prefill with the start states read from a pinned HOST
 * pool (host_state_src, host pointer; src_slot indexes it; -1 = zero state as before).  The
 * states are brought to a staging area behind the workspace proper: when the pool is pinned
 * memory the device can address, by workgroups appended to the first preparation launch (the
 * transfer rides under that launch; only the recurrence needs the states), otherwise by
 * copies on `stream` ahead of the first launch.  The workspace must hold
 * gdn_workspace_bytes_host(...) bytes.  Outputs are bitwise those of gdn_resume_prefill on a
 * device copy of the pool.
 */
int32_t ckpt_fetch_host(const float *host_pool, int64_t host_slot_stride, int32_t host_n_slots,
                        const int32_t *host_ids,
                        float *dev_pool, int64_t dev_slot_stride, int32_t dev_n_slots,
                        const int32_t *dev_ids, int32_t n, int64_t state_elems, void *stream);
int32_t ckpt_spill_host(float *host_pool, int64_t host_slot_stride, int32_t host_n_slots,
                        const int32_t *host_ids,
                        const float *dev_pool, int64_t dev_slot_stride, int32_t dev_n_slots,
                        const int32_t *dev_ids, int32_t n, int64_t state_elems, void *stream);
int64_t gdn_workspace_bytes_host(const gdn_shape *shape, int32_t n_req, int64_t total_tokens,
                                 int32_t n_emit);
int32_t gdn_resume_prefill_host(const gdn_shape *shape,
                                const void *q, const void *k, const void *v,
                                const void *beta, const void *gate,
                                int32_t n_req, const int32_t *cu_seqlens, const int32_t *start_pos,
                                const float *host_state_src, int64_t src_slot_stride,
                                int32_t src_n_slots, const int32_t *src_slot,
                                const int32_t *emit_cu, const int32_t *emit_pos,
                                float *state_dst, int64_t dst_slot_stride, int32_t dst_n_slots,
                                const int32_t *emit_slot,
                                void *o, void *workspace, int64_t workspace_bytes, void *stream);

/*
 * Decode step: one new token per request, the recurrent state updated IN PLACE in its pool
 * slot (same state layout as gdn_resume_prefill; the update is the one-token case of the same
 * recurrence, Sec. 1: a recurrent layer needs only its latest state to go on):
 *     S~ = a S;  u = b (v - S~ k);  S = S~ + u k^T;  o = scale * S q     per (request, layer, value head)
 *   shape       as for gdn_resume_prefill; T_alloc = token rows allocated per layer (>= n_req)
 *   q, k        device [L][T_alloc][H_qk][d_k];  v device [L][T_alloc][H_v][d_v]
 *   beta, gate  device [L][T_alloc][H_v];  row r of every tensor is request r's token
 *   pool        device fp32, slot s at pool + s * slot_stride (floats), read and written
 *   slot        host int32 [n_req] in [0, n_slots), all distinct (two requests may not share a state)
 *   o           device [L][T_alloc][H_v][d_v] in shape->o_dtype, rows 0..n_req-1 written
 * All arithmetic is fp32 on the exactly widened inputs.  Errors as for gdn_resume_prefill
 * (GDN_ERR_SLOT_RANGE, GDN_ERR_SLOT_DUP, GDN_ERR_SEQLENS when n_req > T_alloc, ...); nothing is
 * enqueued when an error is returned.
 */
int32_t gdn_decode_step(const gdn_shape *shape,
                        const void *q, const void *k, const void *v,
                        const void *beta, const void *gate, int32_t n_req,
                        float *pool, int64_t slot_stride, int32_t n_slots, const int32_t *slot,
                        void *o, void *stream);

/*
 * Per-kernel timing for benchmarks (not a step of the method).  While enabled, every
 * gdn_resume_prefill call records HIP events on its stream between its kernel launches (one
 * chunk preparation and one chunk recurrence launch per slab).  gdn_profile_enable(1) clears
 * the totals and starts recording, gdn_profile_enable(0) stops.  gdn_profile_collect waits (on
 * the host) for the recorded events and returns, since recording started: the summed
 * intervals per kernel in milliseconds, the number of calls, and the number of launches of
 * each kernel; any output pointer may be NULL.  The intervals are taken between consecutive
 * events of all calls: meaningful only while calls do not overlap in time.
 */
int32_t gdn_profile_enable(int32_t on);
int32_t gdn_profile_collect(double *prep_ms, double *recur_ms, int64_t *calls,
                            int64_t *prep_launches, int64_t *recur_launches);

/*
 * Machine ceilings for benchmarks (not a step of the method), measured on the current device:
 * the rate of a loop of fp16 matrix instructions (v_mfma_f32_32x32x16_f16, two workgroups of
 * four waves per compute unit) in TFLOP/s, and of a plain 16-byte copy of scratch_bytes / 2
 * bytes from the first half of `scratch` to the second in GB/s (bytes read + written).
 * scratch: device memory, 16-byte aligned, at least 1 MiB, overwritten; a copy figure that
 * means memory bandwidth needs a scratch far larger than the caches (GiB).  Blocks the host
 * until the measurement is done; either output pointer may be NULL.
 */
int32_t gdn_probe_ceilings(void *scratch, int64_t scratch_bytes, double *mfma_f16_tflops,
                           double *copy_gbs, void *stream);

/*
 * Tuning knob (not a step of the method).  gdn_resume_prefill works through a call slab by
 * slab: up to `rounds` consecutive 64-token chunks of every request are prepared, then
 * consumed by the recurrence, then the next slab follows, the states carried in the workspace.
 * rounds > 0 fixes the slab length for later gdn_workspace_bytes / gdn_resume_prefill calls
 * (query the workspace size after setting it); rounds <= 0 restores the automatic choice.
 * Results do not depend on it beyond rounding-order-free bookkeeping: outputs are bitwise
 * the same for every setting.  Returns the previous setting (0 = automatic).
 */
int32_t gdn_tune_slab_rounds(int32_t rounds);

/*
 * Tuning knob (not a step of the method).  Calls with bf16 inputs, d_k = d_v = 128 or 64 and many
 * chains are served by one fused kernel (preparation and recurrence of a chain in one
 * workgroup, no operand image in memory) when the library estimates it to be faster than the
 * two-kernel path.  mode 1 forces the fused kernel wherever it applies, mode 0 forbids it,
 * mode < 0 restores the automatic choice.  Both paths meet the same tolerance; their outputs
 * differ in rounding.  Returns the previous setting (-1 = automatic).
 */
int32_t gdn_tune_fused(int32_t mode);

/*
 * Tuning knob (not a step of the method).  With grouped value heads (H_v / H_qk even) the fused
 * kernel can give two value heads of one query/key head a workgroup of eight waves that reads
 * and stages that head's q and k rows once for both.  mode 1 forces pairs wherever the shape
 * allows them, mode 0 forbids them, mode < 0 restores the automatic choice (pairs at d_k = 128
 * when the call is bound by its volume, not by its longest chain).  Outputs are bitwise the same either way:
 * each head's arithmetic is unchanged.  Returns the previous setting (-1 = automatic).
 */
int32_t gdn_tune_fused_pair(int32_t mode);

/*
 * Tuning knob (not a step of the method).  How many workgroups of the fused kernel may share a
 * compute unit: n >= 1 forces that number (more than fit means as many as fit), n < 1 restores
 * the automatic choice (as many as fit, or one per compute unit when the call is bound by its
 * longest chain: a chain's chunk takes less time on a compute unit of its own).  Outputs are
 * bitwise the same for every setting.  Returns the previous setting (-1 = automatic).
 */
int32_t gdn_tune_fused_per_cu(int32_t n);

/* Version of the library (major * 100 + minor). */
int32_t gdn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* GDN_RESUME_H */
