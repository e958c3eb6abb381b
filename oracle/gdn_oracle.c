/*
 * Oracle for the resume-from-checkpoint recurrent prefill.  TEST INFRASTRUCTURE ONLY:
 * it is called by the tests, by the smoke check and by the benchmark's CPU-baseline
 * leg, never by the product path, and it shares no code with the HIP library.
 *
 * What it computes is the plain definition, token by token, in IEEE double:
 *
 *   - Sec. 1 of the paper: a recurrent layer evolves a fixed-size state
 *     h_t = F(h_{t-1}, x_t); the paper treats F as a black box.  F here is the gated
 *     delta rule of the GatedDeltaNet layer the paper names, per value head, with the
 *     state a d_v x d_k matrix S:
 *         S~  = a_t * S_{t-1}
 *         u_t = b_t * (v_t - S~ k_t)
 *         S_t = S~ + u_t k_t^T          ( = a_t S_{t-1} (I - b_t k_t k_t^T) + b_t v_t k_t^T )
 *         o_t = scale * S_t q_t
 *   - Sec. 3 (problem formulation): a request that overlaps a cached prefix up to depth t
 *     resumes from the deepest checkpoint l(t;C) = max({0} u {c in C : c <= t}) and
 *     replays tokens l+1 .. t; position c means "after consuming tokens 1..c", and
 *     position 0 is the zero state.
 *   - Remark 1: replay from an exact checkpoint equals replay from the start, so the
 *     oracle has no special resume arithmetic: it loads the stored state and runs the
 *     same loop.
 *
 * No chunking, no reordering, no fused steps.  Inputs are the bits the GPU path gets
 * (fp32, or bf16 carried as uint16), widened exactly to double.
 *
 * Parity status: every function here is pinned by tests/test_oracle_pins.py against
 * closed forms, brute-force transition-matrix products written in the test, textbook
 * special cases and the paper's exactness invariant.  The paper prints no worked
 * numeric example for this path, so there is no golden-value pin from the paper.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };

static inline double widen(const void *base, int64_t idx, int dtype)
{
    if (dtype == ORACLE_F32)
        return (double)((const float *)base)[idx];
    uint32_t bits = (uint32_t)((const uint16_t *)base)[idx] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/* Sec. 3: index i of the deepest checkpoint pos[i] <= t, or -1 when none is (the {0}
 * element of the max: resume from the zero state).  Linear scan on purpose. */
int oracle_deepest_ckpt(const int32_t *pos, int M, int32_t t)
{
    int best = -1;
    for (int i = 0; i < M; ++i)
        if (pos[i] <= t && (best < 0 || pos[i] > pos[best]))
            best = i;
    return best;
}

/* Number of threads the prefill below will use (reported next to its timing). */
int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * One call = n_req requests x L layers x H_v value heads, each an independent chain.
 *
 * Token tensors are packed over requests: request r owns packed tokens
 * [cu_seqlens[r], cu_seqlens[r+1]) and they are the tokens at absolute positions
 * start_pos[r]+1 .. start_pos[r]+len_r of its sequence.
 *   q, k  : [L][T_alloc][H_qk][d_k]      v : [L][T_alloc][H_v][d_v]
 *   beta, gate : [L][T_alloc][H_v]       (gate is a_t itself, not its logarithm)
 * Value head h uses query/key head h / (H_v / H_qk).
 * Start state of request r: slot src_slot[r] of state_src ([slot][L][H_v][d_v][d_k]
 * contiguous; fp32 as the checkpoint pool stores it, or double when src_is_f64 is set, which
 * lets a test hand an emitted state back without rounding), or zeros when src_slot[r] < 0.
 * Emissions: request r emits after the tokens at absolute positions
 * emit_pos[emit_cu[r] .. emit_cu[r+1]) (strictly increasing, inside
 * (start_pos[r], start_pos[r]+len_r]); emission e is written to
 * state_out[e] ([n_emit][L][H_v][d_v][d_k], double).
 *   o : [L][T_alloc][H_v][d_v], double.
 * Returns 0, or a negative number for an argument the loop cannot run on.
 */
int oracle_resume_prefill(int L, int H_qk, int H_v, int d_k, int d_v, double scale,
                          int in_dtype, int64_t T_alloc,
                          const void *q, const void *k, const void *v,
                          const void *beta, const void *gate,
                          int n_req, const int32_t *cu_seqlens, const int32_t *start_pos,
                          const void *state_src, int src_is_f64, const int32_t *src_slot,
                          const int32_t *emit_cu, const int32_t *emit_pos,
                          double *state_out, double *o)
{
    if (L <= 0 || H_qk <= 0 || H_v <= 0 || d_k <= 0 || d_v <= 0 || n_req < 0)
        return -1;
    if (H_v % H_qk != 0)
        return -2;
    const int G = H_v / H_qk;
    const int64_t state_elems = (int64_t)d_v * d_k;
    const int64_t slot_elems = (int64_t)L * H_v * state_elems;
    const int64_t n_units = (int64_t)n_req * L * H_v;
    int bad = 0;

#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t unit = 0; unit < n_units; ++unit) {
        const int r = (int)(unit / ((int64_t)L * H_v));
        const int l = (int)((unit / H_v) % L);
        const int h = (int)(unit % H_v);
        const int hq = h / G;

        double *S = (double *)malloc(sizeof(double) * state_elems);
        double *kv = (double *)malloc(sizeof(double) * d_k);
        double *qv = (double *)malloc(sizeof(double) * d_k);
        double *u = (double *)malloc(sizeof(double) * d_v);
        if (!S || !kv || !qv || !u) {
#pragma omp atomic write
            bad = 1;
            free(S); free(kv); free(qv); free(u);
            continue;
        }

        if (src_slot[r] >= 0) {
            const int64_t off = (int64_t)src_slot[r] * slot_elems
                                + ((int64_t)l * H_v + h) * state_elems;
            for (int64_t i = 0; i < state_elems; ++i)
                S[i] = src_is_f64 ? ((const double *)state_src)[off + i]
                                  : (double)((const float *)state_src)[off + i];
        } else {
            for (int64_t i = 0; i < state_elems; ++i)
                S[i] = 0.0;
        }

        int e = emit_cu[r];
        const int e_end = emit_cu[r + 1];
        const int32_t t0 = cu_seqlens[r], t1 = cu_seqlens[r + 1];
        for (int32_t tok = t0; tok < t1; ++tok) {
            const int32_t abs_pos = start_pos[r] + (tok - t0) + 1;
            const int64_t row = (int64_t)l * T_alloc + tok;
            const double a = widen(gate, row * H_v + h, in_dtype);
            const double b = widen(beta, row * H_v + h, in_dtype);
            for (int j = 0; j < d_k; ++j) {
                kv[j] = widen(k, (row * H_qk + hq) * d_k + j, in_dtype);
                qv[j] = widen(q, (row * H_qk + hq) * d_k + j, in_dtype);
            }
            /* S~ = a S */
            for (int64_t i = 0; i < state_elems; ++i)
                S[i] *= a;
            /* u = b (v - S~ k) */
            for (int i = 0; i < d_v; ++i) {
                double dot = 0.0;
                for (int j = 0; j < d_k; ++j)
                    dot += S[(int64_t)i * d_k + j] * kv[j];
                u[i] = b * (widen(v, (row * H_v + h) * d_v + i, in_dtype) - dot);
            }
            /* S = S~ + u k^T */
            for (int i = 0; i < d_v; ++i)
                for (int j = 0; j < d_k; ++j)
                    S[(int64_t)i * d_k + j] += u[i] * kv[j];
            /* o = scale * S q */
            for (int i = 0; i < d_v; ++i) {
                double dot = 0.0;
                for (int j = 0; j < d_k; ++j)
                    dot += S[(int64_t)i * d_k + j] * qv[j];
                o[(row * H_v + h) * d_v + i] = scale * dot;
            }
            /* checkpoint at position c = state after consuming tokens 1..c */
            if (e < e_end && emit_pos[e] == abs_pos) {
                double *dst = state_out + (int64_t)e * slot_elems
                              + ((int64_t)l * H_v + h) * state_elems;
                memcpy(dst, S, sizeof(double) * state_elems);
                ++e;
            }
        }
        free(S); free(kv); free(qv); free(u);
    }
    return bad ? -3 : 0;
}
