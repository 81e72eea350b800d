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
 * Returns 1 and stores s0 = a_j - (u_j + so_i) - b when it fits, else 0 (s0 untouched; s0 may be
 * NULL).  s0 is the printed quantity: the room left for r_i once r_j's own growth over the next
 * so_i iterations and the buffer b are set aside.  r_i's space therefore begins a_j - s0 =
 * u_j + so_i + b tokens into r_j's allocation: after so_i iterations r_j stands b tokens before it. */
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

/* Least-squares fits of the two profiled latency curves (Section 3.5).  n >= 2 points with
 * distinct x; r2 (coefficient of determination in the fitted space) may be NULL.  Return 0, or
 * -1 on bad arguments (n < 2, non-finite values, all x equal; the power law also needs x > 0
 * and y > 0).
 *   kvcp_fit_linear:     y = gamma * x + delta                 (swapping: L_s = gamma_s S + delta_s)
 *   kvcp_fit_power_law:  y = alpha * x^beta, fitted as a line in (ln x, ln y)
 *                        (recomputation with kappa_r = eps_r = 0) */
KVCP_API int kvcp_fit_linear(const double *x, const double *y, int64_t n, double *gamma, double *delta,
                             double *r2);
KVCP_API int kvcp_fit_power_law(const double *x, const double *y, int64_t n, double *alpha, double *beta,
                                double *r2);

/* ---- one scheduler step: batch formation and KVC allocation (Section 3.3.2, 3.3.3, 3.4, 3.5) ---- */

enum { KVCP_WAITING = 0, /* in the queue: new, or preempted earlier and waiting to come back */
       KVCP_RUNNING = 1  /* was in the batch of the iteration that just returned ("returned request") */ };
enum { KVCP_KEEP = 0, KVCP_PREEMPT_SWAP = 1, KVCP_PREEMPT_RECOMPUTE = 2 };
enum { KVCP_CASE_EQUAL = 0, KVCP_CASE_LESS = 1, KVCP_CASE_MORE = 2 };

typedef struct {
    int32_t state;           /* KVCP_WAITING or KVCP_RUNNING */
    int32_t reserved;        /* must be 0 */
    int64_t prompt_len;      /* s^p_i > 0 */
    int64_t est_output_len;  /* s^o_i >= 1, after padding (Section 3.2) */
    int64_t generated;       /* output tokens produced so far */
    int64_t allocated;       /* a_i: KVC tokens allocated to it (0 while waiting) */
    int64_t used;            /* u_i: KVC tokens it occupies (0 while waiting) */
    double remaining_time;   /* RT_i > 0: time left to its TTFT SLO (waiting and never ran) or to its
                                TBT SLO (otherwise) */
    double tbt_slo;          /* its TBT SLO (preemption order) */
} kvcp_request;

typedef struct {
    int64_t unallocated;     /* A'_kvc: KVC tokens allocated to nobody */
    int64_t block_tokens;    /* B: allocation granule in tokens */
    int64_t buffer_tokens;   /* b of the embedding method */
    int64_t token_budget;    /* tokens one iteration should process: a running request counts 1,
                                a waiting one its prompt */
    int64_t token_bucket;    /* bucket width of the preemption order (tokens) */
    int32_t m;               /* proactive allocation: horizon in iterations */
    int32_t n_slo_edges;
    const double *slo_edges; /* TBT-SLO bucket edges of the preemption order (host, ascending) */
    double max_iteration_latency;  /* T_I^max */
    double eps;
    double iter_time_base;       /* iteration latency model base + per_token * tokens, used when */
    double iter_time_per_token;  /* requests are added in the case sum M < A'_kvc */
    double sweet_spot;           /* S_s: sequences longer than this are swapped, others recomputed */
} kvcp_step_params;

typedef struct {
    int32_t in_batch;   /* 1: runs in the next iteration */
    int32_t critical;   /* 1: member of N_w or N_r */
    int32_t preempt;    /* KVCP_KEEP, KVCP_PREEMPT_SWAP or KVCP_PREEMPT_RECOMPUTE */
    int32_t proactive;  /* 1: joined the allocation round through the m-iteration rule */
    int64_t grant;      /* KVC tokens newly allocated to it out of the unallocated KVC */
    int64_t host;       /* index of the running request it is embedded in, else -1 */
    int64_t s0;         /* the s0 of kvcp_embedding_fits (host >= 0 only): its space begins a_host - s0
                           tokens into the host's allocation */
    int64_t lender;     /* index of the running request whose released KVC it will use for its
                           shortfall, else -1 */
    int64_t shortfall;  /* part of its total demand M_i covered neither by its allocation, its grant
                           nor an embedding */
} kvcp_decision;

typedef struct {
    int64_t unallocated_after;  /* A'_kvc left when the step is done */
    int64_t basic_demand;       /* D_kvc of the critical requests that were not embedded */
    int64_t excess;             /* E_kvc = sum M - A'_kvc when the demands were amortised, else 0 */
    int64_t batch_tokens;       /* tokens the formed batch processes */
    int32_t n_preempted;
    int32_t alloc_case;         /* KVCP_CASE_* of the allocation of the remaining KVC */
} kvcp_step_summary;

/*
 * Forms the next batch and allocates KVC, in the order of Section 3.3.2:
 *   1. Running requests with unused allocation stay in the batch.  A running request that has
 *      used up its allocation is critical (N_r) when RT - T_I^max < eps, else it is in N'_r;
 *      waiting requests with RT - T_I^max < eps are critical (N_w).
 *   2. Critical requests, in descending order of their basic requirement (s^p_i + B waiting, B
 *      returned): a waiting one is first tried with the embedding method (host = running request
 *      with unused allocation and the least of it that fits, also after rounding the guest's
 *      space to whole granules of B tokens, see kvcp_embedding_block_range; a host takes one
 *      guest per step);
 *      the others need D_kvc of unallocated KVC.  While A'_kvc < D_kvc, running requests that are
 *      neither critical nor hosts are preempted in the order of Section 3.4, each by swapping if
 *      its occupied KVC exceeds the sweet spot and by recomputation otherwise (Section 3.5); a
 *      victim's allocation returns to A'_kvc.  Then every critical request is granted its basic
 *      requirement (in that order, as long as it fits).
 *   3. The allocation round for the remaining KVC is joined by the critical requests, N'_r,
 *      unfulfilled running requests (a_i < M_i) predicted to finish within m iterations
 *      (Section 3.3.3), and N'_w: waiting requests in ascending RT taken while the batch stays
 *      within the token budget.  Waiting ones are tried with the embedding method first (demand
 *      0 when embedded).  Demands are what is missing to M_i = s^p_i + s^o_i (a request already
 *      beyond its estimate asks for B).  Three cases:
 *        sum = A'_kvc  everybody gets its demand;
 *        sum < A'_kvc  further waiting requests are added in ascending RT while their whole M_i still
 *                      fits and the modelled iteration time stays below every batched request's RT;
 *        sum > A'_kvc  the printed amortisation (kvcp_allocate).
 *      A new request whose share cannot hold its prompt plus B is left out and the round is
 *      repeated without it; alloc_case and excess describe the last round.
 *   4. A batched request with a shortfall borrows: lender = running request in the batch that
 *      finishes (s^o_j - generated_j iterations) no later than the borrower exhausts what it
 *      holds, holds at least the shortfall, and among those finishes latest (then holds least);
 *      a request lends once.
 * req[0..n) and out[0..n) are host arrays; summary may be NULL.  Returns 0, or -1 on invalid
 * arguments (nothing is written then).
 */
KVCP_API int kvcp_schedule_step(const kvcp_request *req, int64_t n, const kvcp_step_params *params,
                                kvcp_decision *out, kvcp_step_summary *summary);

/* Blocks of the host's block list an embedded request occupies: its space begins a_j - s0 tokens
 * into the host's allocation (see kvcp_embedding_fits); it starts at the first block boundary at
 * or after that and spans ceil((sp_i + so_i) / block_size) blocks, so guest and host never share a
 * block.  Returns 0 and stores first / count, or -1 when rounding to blocks pushes it past the
 * host's host_blocks blocks. */
KVCP_API int kvcp_embedding_block_range(int64_t a_j, int64_t s0, int64_t sp_i, int64_t so_i,
                                        int64_t block_size, int64_t host_blocks, int64_t *first,
                                        int64_t *count);

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
