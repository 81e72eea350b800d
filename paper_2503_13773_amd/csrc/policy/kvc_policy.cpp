// Host-side KV-cache scheduling policy of the paper (CPU only); contract in include/kvc_policy.h.
#include "kvc_policy.h"

#include <algorithm>
#include <cmath>
#include <limits>
#include <numeric>
#include <set>
#include <vector>

extern "C" {

double kvcp_confidence(double alpha, double beta, double arrival_rate) {
    if (!(alpha > 0.0 && alpha <= 1.0) || !(beta > 0.0) || !(arrival_rate >= 0.0))
        return std::numeric_limits<double>::quiet_NaN();
    return alpha / (1.0 + beta * arrival_rate);
}

double kvcp_padding(double range, double confidence) {
    if (!(range >= 0.0) || !(confidence >= 0.0 && confidence < 1.0))
        return std::numeric_limits<double>::quiet_NaN();
    return std::sqrt(-(range * range / 2.0) * std::log(1.0 - confidence));
}

double kvcp_estimated_output_len(double predicted, double range, double confidence, int underpredicted) {
    const double t = kvcp_padding(range, confidence);
    if (std::isnan(t) || !(predicted >= 0.0)) return std::numeric_limits<double>::quiet_NaN();
    return std::max(1.0, underpredicted ? predicted + t : predicted - t);
}

int kvcp_embedding_fits(int64_t a_j, int64_t u_j, int64_t sp_i, int64_t so_i, int64_t b, int64_t *s0) {
    if (a_j < 0 || u_j < 0 || u_j > a_j || sp_i < 0 || so_i < 0 || b < 0) return 0;
    if (a_j - (u_j + so_i) - (sp_i + so_i) < b) return 0;
    if (s0) *s0 = a_j - (u_j + so_i) - b;
    return 1;
}

int64_t kvcp_embedding_choose(const int64_t *a, const int64_t *u, int64_t n_running, int64_t sp_i,
                              int64_t so_i, int64_t b, int64_t *s0) {
    if (n_running < 0 || (n_running > 0 && (!a || !u))) return -1;
    int64_t best = -1, best_remaining = 0, best_s0 = 0;
    for (int64_t j = 0; j < n_running; ++j) {
        int64_t start;
        if (!kvcp_embedding_fits(a[j], u[j], sp_i, so_i, b, &start)) continue;
        const int64_t remaining = a[j] - u[j];
        if (best < 0 || remaining < best_remaining) {
            best = j;
            best_remaining = remaining;
            best_s0 = start;
        }
    }
    if (best >= 0 && s0) *s0 = best_s0;
    return best;
}

int kvcp_is_critical(double remaining_time, double max_iteration_latency, double eps) {
    return (remaining_time - max_iteration_latency) < eps ? 1 : 0;
}

int64_t kvcp_basic_demand(const int64_t *sp_critical_waiting, int64_t n_waiting, int64_t n_returned, int64_t B) {
    if (n_waiting < 0 || n_returned < 0 || B < 0 || (n_waiting > 0 && !sp_critical_waiting)) return -1;
    int64_t d = n_returned * B;
    for (int64_t i = 0; i < n_waiting; ++i) {
        if (sp_critical_waiting[i] < 0) return -1;
        d += sp_critical_waiting[i] + B;
    }
    return d;
}

int kvcp_allocate(const int64_t *M, const double *RT, const int64_t *sp, int64_t n, int64_t A_avail,
                  int64_t *A_out, int64_t *slack) {
    if (n < 0 || A_avail < 0 || (n > 0 && (!M || !A_out))) return -1;
    int64_t total = 0;
    for (int64_t i = 0; i < n; ++i) {
        if (M[i] < 0) return -1;
        total += M[i];
    }
    if (total <= A_avail) {
        for (int64_t i = 0; i < n; ++i) A_out[i] = M[i];
        if (slack) *slack = A_avail - total;
        return 0;
    }
    if (!RT || !sp) return -1;
    double sum_rt = 0.0, sum_sp = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        if (M[i] == 0) continue;
        if (!(RT[i] > 0.0) || sp[i] <= 0) return -1;
        sum_rt += RT[i];
        sum_sp += double(sp[i]);
    }
    std::vector<double> w(n, 0.0);
    double sum_w = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        if (M[i] == 0) continue;
        w[i] = (RT[i] / sum_rt) * (double(sp[i]) / sum_sp);
        sum_w += w[i];
    }
    for (int64_t i = 0; i < n; ++i) {
        const int64_t share = M[i] == 0 ? 0 : int64_t(std::floor(double(A_avail) * (w[i] / sum_w)));
        A_out[i] = std::min(share, M[i]);
    }
    if (slack) *slack = -(total - A_avail);
    return 0;
}

int kvcp_preemption_order(const double *tbt_slo, const int64_t *remaining_tokens,
                          const int64_t *occupied_kvc, int64_t n, const double *slo_edges,
                          int32_t n_edges, int64_t token_bucket, int64_t *order_out) {
    if (n < 0 || n_edges < 0 || token_bucket <= 0 || (n_edges > 0 && !slo_edges)) return -1;
    if (n > 0 && (!tbt_slo || !remaining_tokens || !occupied_kvc || !order_out)) return -1;
    for (int32_t k = 1; k < n_edges; ++k)
        if (!(slo_edges[k] > slo_edges[k - 1])) return -1;
    auto slo_bucket = [&](double v) {
        int32_t k = 0;
        while (k < n_edges && slo_edges[k] <= v) ++k;
        return k;
    };
    std::vector<int64_t> idx(n);
    std::iota(idx.begin(), idx.end(), int64_t(0));
    std::stable_sort(idx.begin(), idx.end(), [&](int64_t x, int64_t y) {
        const int32_t bx = slo_bucket(tbt_slo[x]), by = slo_bucket(tbt_slo[y]);
        if (bx != by) return bx > by;                                  // looser SLO first
        const int64_t rx = remaining_tokens[x] / token_bucket, ry = remaining_tokens[y] / token_bucket;
        if (rx != ry) return rx > ry;                                  // longer remaining time first
        return occupied_kvc[x] < occupied_kvc[y];                      // less KVC to move first
    });
    std::copy(idx.begin(), idx.end(), order_out);
    return 0;
}

double kvcp_sweet_spot(double gamma_s, double delta_s, double alpha_r, double beta_r, double kappa_r,
                       double eps_r, double s_max) {
    auto f = [&](double s) {
        return (alpha_r * std::pow(s, beta_r) + kappa_r * s + eps_r) - (gamma_s * s + delta_s);
    };
    double lo = 1.0, hi = s_max;
    if (!(hi > lo)) return std::numeric_limits<double>::quiet_NaN();
    if (f(lo) >= 0.0) return 0.0;
    if (f(hi) < 0.0) return std::numeric_limits<double>::infinity();
    for (int it = 0; it < 200; ++it) {
        const double mid = 0.5 * (lo + hi);
        if (f(mid) < 0.0) lo = mid; else hi = mid;
    }
    return 0.5 * (lo + hi);
}

int kvcp_choose_swap(double seq_len, double sweet_spot) { return seq_len > sweet_spot ? 1 : 0; }

}  // extern "C"

struct kvcp_block_manager {
    int64_t num_blocks;
    int64_t first_reserved;          // ids >= first_reserved belong to the reserved pool
    std::set<int32_t> free_general;  // ordered: lowest id first
    std::set<int32_t> free_reserved;
};

extern "C" {

kvcp_block_manager *kvcp_bm_create(int64_t num_blocks, int64_t reserved_blocks) {
    if (num_blocks <= 0 || reserved_blocks < 0 || reserved_blocks > num_blocks ||
        num_blocks > std::numeric_limits<int32_t>::max())
        return nullptr;
    auto *bm = new kvcp_block_manager;
    bm->num_blocks = num_blocks;
    bm->first_reserved = num_blocks - reserved_blocks;
    for (int64_t i = 0; i < bm->first_reserved; ++i) bm->free_general.insert(int32_t(i));
    for (int64_t i = bm->first_reserved; i < num_blocks; ++i) bm->free_reserved.insert(int32_t(i));
    return bm;
}

void kvcp_bm_destroy(kvcp_block_manager *bm) { delete bm; }
int64_t kvcp_bm_free_general(const kvcp_block_manager *bm) { return bm ? int64_t(bm->free_general.size()) : -1; }
int64_t kvcp_bm_free_reserved(const kvcp_block_manager *bm) { return bm ? int64_t(bm->free_reserved.size()) : -1; }

static int take(std::set<int32_t> &pool, int64_t n, int32_t *ids_out) {
    if (n < 0 || (n > 0 && !ids_out) || int64_t(pool.size()) < n) return -1;
    for (int64_t i = 0; i < n; ++i) {
        ids_out[i] = *pool.begin();
        pool.erase(pool.begin());
    }
    return 0;
}

int kvcp_bm_allocate(kvcp_block_manager *bm, int64_t n, int32_t *ids_out) {
    return bm ? take(bm->free_general, n, ids_out) : -1;
}
int kvcp_bm_allocate_reserved(kvcp_block_manager *bm, int64_t n, int32_t *ids_out) {
    return bm ? take(bm->free_reserved, n, ids_out) : -1;
}

int kvcp_bm_release(kvcp_block_manager *bm, const int32_t *ids, int64_t n) {
    if (!bm || n < 0 || (n > 0 && !ids)) return -1;
    std::set<int32_t> seen;
    for (int64_t i = 0; i < n; ++i) {
        const int32_t id = ids[i];
        if (id < 0 || id >= bm->num_blocks || !seen.insert(id).second) return -1;
        if (bm->free_general.count(id) || bm->free_reserved.count(id)) return -1;
    }
    for (int64_t i = 0; i < n; ++i)
        (ids[i] >= bm->first_reserved ? bm->free_reserved : bm->free_general).insert(ids[i]);
    return 0;
}

}  // extern "C"
