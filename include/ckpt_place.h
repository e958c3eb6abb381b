/*
 * Placement of recurrent-state checkpoints on a cached prefix: host code, off the serving
 * path (Theorem 2 of the paper and the remark after it: a schedule is computed offline and
 * refreshed when the overlap histogram is updated).  Plain C ABI, host pointers only, no
 * GPU work, no allocation visible to the caller except the histogram handle.
 *
 * Notation (Sec. 3): cached prefix of N tokens, budget of M checkpoints, positions
 * 1 <= c_1 < ... < c_M <= N, a checkpoint at c holds the state after token c; overlap depth
 * t in 1..N has mass p_t (array p[t-1]; weights need not be normalised, must be >= 0);
 * l(t; C) = deepest checkpoint <= t (0 if none), recomputation r = t - l.
 *
 * Every function returns a count or GDN_OK (0) on success and a negative gdn_resume.h error
 * code on bad arguments (GDN_ERR_NULL, GDN_ERR_COUNT for sizes out of range,
 * GDN_ERR_WORKSPACE when `capacity` is too small, GDN_ERR_EMIT for positions that are not
 * strictly increasing inside [1, N]).
 */
#ifndef CKPT_PLACE_H
#define CKPT_PLACE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Table 1, "Balanced": pos[i-1] = floor(i (N+1) / (M+1)), i = 1..M (needs M <= N).  Returns M. */
int32_t ckpt_place_balanced(int32_t N, int32_t M, int32_t *pos);

/* Table 1, "Block": B, 2B, ..., floor(N/B) B.  Returns the count. */
int32_t ckpt_place_block(int32_t N, int32_t B, int32_t *pos, int32_t capacity);

/* Table 1, "sqrt(L)": multiples of floor(sqrt(N)) up to N.  Returns the count. */
int32_t ckpt_place_sqrt(int32_t N, int32_t *pos, int32_t capacity);

/*
 * Sec. 5 baselines, "Logarithmic": gap sizes that grow exponentially from the beginning of
 * the prefix.  The paper gives neither base nor unit; this build doubles the gap, starting
 * at `unit` tokens: positions unit (2^i - 1), i = 1, 2, ..., while <= N and at most M.
 * Returns the count.
 */
int32_t ckpt_place_log(int32_t N, int32_t unit, int32_t M, int32_t *pos);

/*
 * Sec. 5: every position is clipped to a block boundary (floor to a multiple of B);
 * positions that become 0 or repeat are dropped.  pos: n strictly increasing positions;
 * out: room for n.  Returns the count kept.
 */
int32_t ckpt_clip_to_blocks(const int32_t *pos, int32_t n, int32_t B, int32_t *out);

/*
 * Sec. 3: expected recomputation E[r(T; C)] = sum_t p_t (t - l(t; C)) and the no-cache work
 * R_nc = sum_t p_t t, from which Savings = 1 - E[r]/R_nc and Reduction = R_nc/E[r]
 * (reduction is +inf when E[r] = 0).  pos may be NULL when n = 0.  Any output may be NULL.
 */
int32_t ckpt_expected_recompute(const double *p, int32_t N, const int32_t *pos, int32_t n,
                                double *expected, double *no_cache, double *savings,
                                double *reduction);

/*
 * Theorem 2: the checkpoint set of at most M positions that minimises E[r(T; C)] for the
 * masses p, by the dynamic program dp[m, j] = min_s dp[m-1, s-1] + w(s, j) evaluated with the
 * monotone convex hull trick, O(N M) time, O(N M) int32 memory for the back-pointers.
 * pos: room for M; receives the positions in increasing order.  cost (may be NULL): the
 * minimum.  Returns the number of positions placed (<= M; fewer when extra checkpoints
 * cannot lower the cost).  Ties between equally good sets are broken arbitrarily.
 */
int32_t ckpt_place_dp(const double *p, int32_t N, int32_t M, int32_t *pos, double *cost);

/*
 * Sec. 4.2 / Sec. 5 "Our method": exponentially weighted overlap histogram
 * p^_t = (1-g)/(1-g^n) sum_s g^(n-s) e_{T_s} over the n depths observed so far.
 * ckpt_hist_create returns a handle (NULL on bad arguments: N < 1, gamma outside (0, 1]);
 * gamma = 1 gives the plain empirical histogram.  ckpt_hist_observe records one depth in
 * 1..N and returns the number of observations so far.  ckpt_hist_get writes the N masses
 * (they sum to 1; all zero before the first observation).  ckpt_hist_solve runs
 * ckpt_place_dp on the current histogram and, when B > 1, clips the result to blocks;
 * returns the count.  The handle is not thread safe; destroy it with ckpt_hist_destroy.
 */
typedef struct ckpt_hist ckpt_hist;
ckpt_hist *ckpt_hist_create(int32_t N, double gamma);
void ckpt_hist_destroy(ckpt_hist *h);
int64_t ckpt_hist_observe(ckpt_hist *h, int32_t t);
int32_t ckpt_hist_get(const ckpt_hist *h, double *p);
int32_t ckpt_hist_solve(const ckpt_hist *h, int32_t M, int32_t B, int32_t *pos, double *cost);

/*
 * Sec. 5, "Our method": the online loop around the histogram.  Every observed overlap depth
 * updates the exponentially weighted histogram (the paper uses gamma = 0.99); after every
 * `period` observations (10 in the paper) the dynamic program is solved again on the current
 * estimate with budget M and the result clipped to blocks of B (1 = no clipping).
 * ckpt_online_create returns NULL on bad arguments (N, M, B, period < 1, gamma outside (0, 1]).
 * ckpt_online_observe returns 1 when this observation triggered a re-solve (the schedule may
 * have changed), 0 otherwise, negative on error (depth outside 1..N: GDN_ERR_COUNT).
 * ckpt_online_schedule copies the current schedule (empty before the first re-solve) into pos
 * (room for `capacity`) and returns its length.  ckpt_online_histogram lends the histogram for
 * ckpt_hist_get.  Not thread safe.
 */
typedef struct ckpt_online ckpt_online;
ckpt_online *ckpt_online_create(int32_t N, int32_t M, int32_t B, double gamma, int32_t period);
void ckpt_online_destroy(ckpt_online *o);
int32_t ckpt_online_observe(ckpt_online *o, int32_t t);
int32_t ckpt_online_schedule(const ckpt_online *o, int32_t *pos, int32_t capacity);
const ckpt_hist *ckpt_online_histogram(const ckpt_online *o);

#ifdef __cplusplus
}
#endif
#endif /* CKPT_PLACE_H */
