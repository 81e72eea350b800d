/*
 * kvc_policy.h - C ABI of the host-side KV-cache scheduling policy of the paper (CPU only).
 *
 * These are the closed-form pieces of the method the device path serves: confidence-based
 * padding (Section 3.2), the embedding method and the SLO-aware KVC allocation (Section 3.3),
 * the preemption order (Section 3.4) and the swap-or-recompute choice (Section 3.5), plus a
 * block manager with a globally reserved pool (Section 3.3.3) that produces the block ids the
 * device calls (kvc.h) consume.  Everything here is plain host arithmetic: no GPU, no I/O.
 *
 * All pointers are host memory owned by the caller; arrays are read during the call only.
 * Functions that can fail return a negative value (see each); the others are total.
 * Lengths and KVC amounts are in tokens unless a name says "blocks".
 */
#ifndef KVC_POLICY_H
#define KVC_POLICY_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define KVCP_API __attribute__((visibility("default")))

/* ---- confidence-based padding (Section 3.2) ---- */

/* Eq. 4: c = alpha / (1 + beta * lambda), 0 < alpha <= 1, beta > 0, lambda >= 0 the request
 * arrival rate.  Returns NaN for arguments outside those ranges. */
KVCP_API double kvcp_confidence(double alpha, double beta, double arrival_rate);

/* Eq. 3: padding t = sqrt( -(range^2 / 2) * ln(1 - c) ), range = b_i - a_i the spread of output
 * lengths among the predicted values, 0 <= c < 1.  Returns NaN outside those ranges. */
KVCP_API double kvcp_padding(double range, double confidence);

/* Estimated output length s^o: the padding is added when the predictor's deviation direction
 * says "underpredicted" (nonzero) and subtracted otherwise; never below 1 token. */
KVCP_API double kvcp_estimated_output_len(double predicted, double range, double confidence,
                                          int underpredicted);

/* ---- embedding method (Section 3.3.1) ---- */

/* Request i (prompt sp_i, estimated output so_i) fits into running request j's allocated but
 * unused KVC (allocated a_j, used u_j) iff a_j - (u_j + so_i) - (sp_i + so_i) >= b.
 * Returns 1 and stores the start offset s0 = a_j - (u_j + so_i) - b (tokens from the start of
 * r_j's allocation) when it fits, else 0 (s0 untouched).  s0 may be NULL. */
KVCP_API int kvcp_embedding_fits(int64_t a_j, int64_t u_j, int64_t sp_i, int64_t so_i, int64_t b,
                                 int64_t *s0);

/* Among n_running requests (allocated a[], used u[]) pick the host with the minimum remaining
 * allocated KVC a_j - u_j that request i fits into (ties: lowest index).  Returns its index and
 * stores s0, or -1 when none fits. */
KVCP_API int64_t kvcp_embedding_choose(const int64_t *a, const int64_t *u, int64_t n_running,
                                       int64_t sp_i, int64_t so_i, int64_t b, int64_t *s0);

/* ---- request selection and KVC allocation (Section 3.3.2) ---- */

/* A request is critical when RT - T_I^max < eps (RT: remaining time to its TTFT or TBT SLO,
 * T_I^max: the maximum iteration latency seen so far). */
KVCP_API int kvcp_is_critical(double remaining_time, double max_iteration_latency, double eps);

/* Basic KVC demand of the critical requests: D = sum over critical waiting requests of
 * (s^p_i + B) + (number of critical returned requests) * B. */
KVCP_API int64_t kvcp_basic_demand(const int64_t *sp_critical_waiting, int64_t n_waiting,
                                   int64_t n_returned, int64_t B);

/* Distribute the unallocated KVC A' among n requests with total demands M[]:
 *   sum M <= A'  : every request gets its demand; *slack = A' - sum M (room to batch more requests);
 *   sum M >  A'  : the excess is amortised with the printed weights
 *                  w_i = RT_i / sum RT * s^p_i / sum s^p,  A_i = floor(A' * w_i / sum w), capped at
 *                  M_i; *slack = -(sum M - A') (the excess E_kvc, negative).
 * Requests embedded elsewhere are passed with M_i = 0 and receive 0.  Returns 0, or -1 when an
 * argument is invalid (n < 0, negative amounts, non-positive RT or s^p among requests with M_i > 0
 * in the amortised case).  slack may be NULL. */
KVCP_API int kvcp_allocate(const int64_t *M, const double *RT, const int64_t *sp, int64_t n,
                           int64_t A_avail, int64_t *A_out, int64_t *slack);

/* ---- preemption policy (Section 3.4) ---- */

/* Order n requests for preemption: descending TBT-SLO bucket (bucket edges slo_edges[0..n_edges):
 * a value v falls in bucket k = number of edges <= v), then descending bucket of remaining
 * predicted output tokens (bucket width token_bucket), then ascending occupied KVC; ties by
 * index.  order_out[0] is the first request to preempt.  Returns 0 or -1 on bad arguments. */
KVCP_API int kvcp_preemption_order(const double *tbt_slo, const int64_t *remaining_tokens,
                                   const int64_t *occupied_kvc, int64_t n, const double *slo_edges,
                                   int32_t n_edges, int64_t token_bucket, int64_t *order_out);

/* ---- preemption strategy (Section 3.5) ---- */

/* Sequence length S_s with L_r(S) = L_s(S), L_r(S) = alpha_r S^beta_r + kappa_r S + eps_r,
 * L_s(S) = gamma_s S + delta_s, searched on [1, s_max] by bisection.  Returns 0 when swapping is
 * already cheaper at S = 1 and +inf when recomputation stays cheaper up to s_max. */
KVCP_API double kvcp_sweet_spot(double gamma_s, double delta_s, double alpha_r, double beta_r,
                                double kappa_r, double eps_r, double s_max);

/* 1 = swap, 0 = recompute: swap iff the sequence length exceeds the sweet spot. */
KVCP_API int kvcp_choose_swap(double seq_len, double sweet_spot);

/* ---- block manager with a globally reserved pool (Section 3.3.3) ---- */

typedef struct kvcp_block_manager kvcp_block_manager;

/* Blocks 0 .. num_blocks-1; the last reserved_blocks of them form the shared reserved pool that
 * ordinary allocation never touches.  NULL on bad arguments. */
KVCP_API kvcp_block_manager *kvcp_bm_create(int64_t num_blocks, int64_t reserved_blocks);
KVCP_API void kvcp_bm_destroy(kvcp_block_manager *bm);
KVCP_API int64_t kvcp_bm_free_general(const kvcp_block_manager *bm);
KVCP_API int64_t kvcp_bm_free_reserved(const kvcp_block_manager *bm);
/* All-or-nothing allocation of n blocks from the general pool (lowest free ids first) or from
 * the reserved pool (used on allocation failure).  Returns 0, or -1 if fewer than n are free
 * (nothing is taken then). */
KVCP_API int kvcp_bm_allocate(kvcp_block_manager *bm, int64_t n, int32_t *ids_out);
KVCP_API int kvcp_bm_allocate_reserved(kvcp_block_manager *bm, int64_t n, int32_t *ids_out);
/* Return blocks to the pool they belong to.  Returns -1 (and releases nothing) if an id is out
 * of range, listed twice, or not currently allocated. */
KVCP_API int kvcp_bm_release(kvcp_block_manager *bm, const int32_t *ids, int64_t n);

#ifdef __cplusplus
}
#endif
#endif /* KVC_POLICY_H */
