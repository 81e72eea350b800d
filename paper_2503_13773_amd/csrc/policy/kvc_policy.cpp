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

// Ordinary least squares of y on x; also the coefficient of determination.
static int fit_line(const std::vector<double> &x, const std::vector<double> &y, double *slope,
                    double *intercept, double *r2) {
    const size_t n = x.size();
    double mx = 0.0, my = 0.0;
    for (size_t i = 0; i < n; ++i) {
        if (!std::isfinite(x[i]) || !std::isfinite(y[i])) return -1;
        mx += x[i];
        my += y[i];
    }
    mx /= double(n);
    my /= double(n);
    double sxx = 0.0, sxy = 0.0, syy = 0.0;
    for (size_t i = 0; i < n; ++i) {
        sxx += (x[i] - mx) * (x[i] - mx);
        sxy += (x[i] - mx) * (y[i] - my);
        syy += (y[i] - my) * (y[i] - my);
    }
    if (!(sxx > 0.0)) return -1;
    const double k = sxy / sxx, c = my - k * mx;
    if (slope) *slope = k;
    if (intercept) *intercept = c;
    if (r2) {
        double sse = 0.0;
        for (size_t i = 0; i < n; ++i) {
            const double e = y[i] - (k * x[i] + c);
            sse += e * e;
        }
        *r2 = syy > 0.0 ? 1.0 - sse / syy : 1.0;
    }
    return 0;
}

int kvcp_fit_linear(const double *x, const double *y, int64_t n, double *gamma, double *delta, double *r2) {
    if (n < 2 || !x || !y || !gamma || !delta) return -1;
    return fit_line(std::vector<double>(x, x + n), std::vector<double>(y, y + n), gamma, delta, r2);
}

int kvcp_fit_power_law(const double *x, const double *y, int64_t n, double *alpha, double *beta, double *r2) {
    if (n < 2 || !x || !y || !alpha || !beta) return -1;
    std::vector<double> lx(n), ly(n);
    for (int64_t i = 0; i < n; ++i) {
        if (!(x[i] > 0.0) || !(y[i] > 0.0)) return -1;
        lx[i] = std::log(x[i]);
        ly[i] = std::log(y[i]);
    }
    double k, c;
    if (fit_line(lx, ly, &k, &c, r2) != 0) return -1;
    *beta = k;
    *alpha = std::exp(c);
    return 0;
}

int kvcp_embedding_block_range(int64_t a_j, int64_t s0, int64_t sp_i, int64_t so_i, int64_t block_size,
                               int64_t host_blocks, int64_t *first, int64_t *count) {
    if (a_j < 0 || s0 < 0 || s0 > a_j || sp_i < 0 || so_i < 0 || block_size <= 0 || host_blocks < 0 || !first ||
        !count)
        return -1;
    const int64_t f = (a_j - s0 + block_size - 1) / block_size;
    const int64_t c = (sp_i + so_i + block_size - 1) / block_size;
    if (f + c > host_blocks) return -1;
    *first = f;
    *count = c;
    return 0;
}

int kvcp_schedule_step(const kvcp_request *req, int64_t n, const kvcp_step_params *p, kvcp_decision *out,
                       kvcp_step_summary *summary) {
    if (n < 0 || !p || (n > 0 && (!req || !out))) return -1;
    if (p->unallocated < 0 || p->block_tokens <= 0 || p->buffer_tokens < 0 || p->token_budget < 0 ||
        p->token_bucket <= 0 || p->m < 0 || p->n_slo_edges < 0 || (p->n_slo_edges > 0 && !p->slo_edges) ||
        !(p->iter_time_base >= 0.0) || !(p->iter_time_per_token >= 0.0) || std::isnan(p->sweet_spot) ||
        std::isnan(p->max_iteration_latency) || std::isnan(p->eps))
        return -1;
    for (int64_t i = 0; i < n; ++i) {
        const kvcp_request &r = req[i];
        if ((r.state != KVCP_WAITING && r.state != KVCP_RUNNING) || r.reserved != 0 || r.prompt_len <= 0 ||
            r.est_output_len < 1 || r.generated < 0 || r.allocated < 0 || r.used < 0 || r.used > r.allocated ||
            !(r.remaining_time > 0.0) || std::isnan(r.tbt_slo))
            return -1;
        if (r.state == KVCP_WAITING && (r.allocated != 0 || r.used != 0)) return -1;
    }
    const int64_t B = p->block_tokens;
    int64_t avail = p->unallocated;
    std::vector<kvcp_decision> d(n);
    for (auto &x : d) x = kvcp_decision{0, 0, KVCP_KEEP, 0, 0, -1, 0, -1, 0};
    auto total_demand = [&](int64_t i) { return req[i].prompt_len + req[i].est_output_len; };
    auto critical_time = [&](int64_t i) {
        return kvcp_is_critical(req[i].remaining_time, p->max_iteration_latency, p->eps) != 0;
    };

    // ---- 1. who is where
    std::vector<int64_t> crit, nr_prime, waiting_rest;
    std::vector<char> is_host(n, 0), out_of_kvc(n, 0);
    for (int64_t i = 0; i < n; ++i) {
        if (req[i].state == KVCP_RUNNING) {
            d[i].in_batch = 1;
            if (req[i].used >= req[i].allocated) {
                out_of_kvc[i] = 1;
                if (critical_time(i)) { d[i].critical = 1; crit.push_back(i); }
                else nr_prime.push_back(i);
            }
        } else if (critical_time(i)) {
            d[i].critical = 1;
            crit.push_back(i);
        } else {
            waiting_rest.push_back(i);
        }
    }
    auto basic = [&](int64_t i) { return req[i].state == KVCP_WAITING ? req[i].prompt_len + B : B; };
    std::stable_sort(crit.begin(), crit.end(), [&](int64_t x, int64_t y) { return basic(x) > basic(y); });
    std::stable_sort(waiting_rest.begin(), waiting_rest.end(),
                     [&](int64_t x, int64_t y) { return req[x].remaining_time < req[y].remaining_time; });

    // Embedding method for waiting request i: host = running request with unused allocation, not out
    // of KVC, not preempted, not a host already, with the least remaining allocation that fits.
    auto try_embed = [&](int64_t i) {
        int64_t best = -1, best_rem = 0, best_s0 = 0;
        for (int64_t j = 0; j < n; ++j) {
            if (req[j].state != KVCP_RUNNING || out_of_kvc[j] || is_host[j] || d[j].preempt != KVCP_KEEP) continue;
            int64_t s0;
            if (!kvcp_embedding_fits(req[j].allocated, req[j].used, req[i].prompt_len, req[i].est_output_len,
                                     p->buffer_tokens, &s0))
                continue;
            int64_t first, count;  // KVC is handed out in granules of B tokens: the guest must fit in whole ones
            if (kvcp_embedding_block_range(req[j].allocated, s0, req[i].prompt_len, req[i].est_output_len, B,
                                           req[j].allocated / B, &first, &count) != 0)
                continue;
            const int64_t rem = req[j].allocated - req[j].used;
            if (best < 0 || rem < best_rem) { best = j; best_rem = rem; best_s0 = s0; }
        }
        if (best < 0) return false;
        is_host[best] = 1;
        d[i].host = best;
        d[i].s0 = best_s0;
        d[i].in_batch = 1;
        return true;
    };

    // ---- 2. critical requests: embedding, preemptions up to the basic demand, basic grants
    std::vector<int64_t> crit_unembedded;
    int64_t D = 0;
    for (int64_t i : crit) {
        if (req[i].state == KVCP_WAITING && try_embed(i)) continue;
        crit_unembedded.push_back(i);
        D += basic(i);
    }
    int32_t n_preempted = 0;
    if (avail < D) {
        std::vector<int64_t> cand;
        for (int64_t j = 0; j < n; ++j)
            if (req[j].state == KVCP_RUNNING && !d[j].critical && !is_host[j]) cand.push_back(j);
        std::vector<double> slo(cand.size());
        std::vector<int64_t> rem(cand.size()), occ(cand.size()), order(cand.size());
        for (size_t k = 0; k < cand.size(); ++k) {
            slo[k] = req[cand[k]].tbt_slo;
            rem[k] = std::max<int64_t>(0, req[cand[k]].est_output_len - req[cand[k]].generated);
            occ[k] = req[cand[k]].used;
        }
        if (!cand.empty() &&
            kvcp_preemption_order(slo.data(), rem.data(), occ.data(), int64_t(cand.size()), p->slo_edges,
                                  p->n_slo_edges, p->token_bucket, order.data()) != 0)
            return -1;
        for (size_t k = 0; k < cand.size() && avail < D; ++k) {
            const int64_t v = cand[order[k]];
            d[v].preempt = kvcp_choose_swap(double(req[v].used), p->sweet_spot) ? KVCP_PREEMPT_SWAP
                                                                               : KVCP_PREEMPT_RECOMPUTE;
            d[v].in_batch = 0;
            avail += req[v].allocated;
            ++n_preempted;
        }
    }
    for (int64_t i : crit_unembedded) {
        if (basic(i) <= avail) {
            d[i].grant = basic(i);
            d[i].in_batch = 1;
            avail -= basic(i);
        } else {
            d[i].in_batch = 0;  // not even the victims' KVC covers it: it waits
        }
    }

    // ---- 3. the allocation round for the remaining KVC
    int64_t batch_tokens = 0;
    for (int64_t i = 0; i < n; ++i)
        if (d[i].in_batch) batch_tokens += req[i].state == KVCP_RUNNING ? 1 : req[i].prompt_len;
    std::vector<int64_t> round;  // members with a demand (possibly 0)
    std::vector<int64_t> demand(n, 0);
    for (int64_t i : crit) {
        if (!d[i].in_batch) continue;
        if (d[i].host >= 0) continue;  // embedded: whole demand placed in the host
        demand[i] = std::max<int64_t>(0, total_demand(i) - req[i].allocated - d[i].grant);
        round.push_back(i);
    }
    for (int64_t i : nr_prime) {
        if (d[i].preempt != KVCP_KEEP) continue;
        const int64_t missing = total_demand(i) - req[i].allocated;
        demand[i] = missing > 0 ? missing : B;
        round.push_back(i);
    }
    for (int64_t i = 0; i < n; ++i) {  // proactive allocation: unfulfilled, about to finish
        if (req[i].state != KVCP_RUNNING || out_of_kvc[i] || d[i].preempt != KVCP_KEEP) continue;
        const int64_t left = req[i].est_output_len - req[i].generated;
        if (req[i].allocated < total_demand(i) && left >= 0 && left <= p->m) {
            d[i].proactive = 1;
            demand[i] = total_demand(i) - req[i].allocated;
            round.push_back(i);
        }
    }
    size_t next_waiting = 0;
    auto add_waiting = [&](int64_t i) {
        d[i].in_batch = 1;
        batch_tokens += req[i].prompt_len;
        if (!try_embed(i)) demand[i] = total_demand(i);
        round.push_back(i);
    };
    for (; next_waiting < waiting_rest.size(); ++next_waiting) {  // N'_w: up to the token budget
        const int64_t i = waiting_rest[next_waiting];
        if (batch_tokens + req[i].prompt_len > p->token_budget) break;
        add_waiting(i);
    }
    auto sum_demand = [&]() {
        int64_t t = 0;
        for (int64_t i : round) t += demand[i];
        return t;
    };
    int64_t total = sum_demand();
    int32_t alloc_case = total == avail ? KVCP_CASE_EQUAL : total < avail ? KVCP_CASE_LESS : KVCP_CASE_MORE;
    if (alloc_case == KVCP_CASE_LESS) {
        double min_rt = std::numeric_limits<double>::infinity();
        for (int64_t i = 0; i < n; ++i)
            if (d[i].in_batch) min_rt = std::min(min_rt, req[i].remaining_time);
        for (; next_waiting < waiting_rest.size(); ++next_waiting) {
            const int64_t i = waiting_rest[next_waiting];
            if (total + total_demand(i) > avail) break;
            const double t_iter = p->iter_time_base + p->iter_time_per_token * double(batch_tokens + req[i].prompt_len);
            if (t_iter > std::min(min_rt, req[i].remaining_time)) break;
            add_waiting(i);
            min_rt = std::min(min_rt, req[i].remaining_time);
            total = sum_demand();
        }
    }
    // A new request must at least hold its prompt and one granule: one whose share is smaller is
    // left out and the round is repeated without it.
    int64_t excess = 0;
    const int64_t round_avail = avail;
    std::vector<int64_t> share(n, 0);
    for (bool again = true; again && !round.empty();) {
        again = false;
        std::vector<int64_t> M(round.size()), sp(round.size()), A(round.size());
        std::vector<double> RT(round.size());
        for (size_t k = 0; k < round.size(); ++k) {
            M[k] = demand[round[k]];
            sp[k] = req[round[k]].prompt_len;
            RT[k] = req[round[k]].remaining_time;
        }
        int64_t slack = 0;
        if (kvcp_allocate(M.data(), RT.data(), sp.data(), int64_t(round.size()), round_avail, A.data(), &slack) != 0)
            return -1;
        excess = slack < 0 ? -slack : 0;
        alloc_case = slack == 0 ? KVCP_CASE_EQUAL : slack > 0 ? KVCP_CASE_LESS : KVCP_CASE_MORE;
        std::vector<int64_t> kept;
        for (size_t k = 0; k < round.size(); ++k) {
            const int64_t i = round[k];
            share[i] = A[k];
            if (req[i].state == KVCP_WAITING && d[i].host < 0 && d[i].grant + A[k] < req[i].prompt_len + B) {
                batch_tokens -= req[i].prompt_len;
                d[i].in_batch = 0;
                share[i] = 0;
                again = true;
            } else {
                kept.push_back(i);
            }
        }
        round.swap(kept);
    }
    for (int64_t i : round) {
        d[i].grant += share[i];
        avail -= share[i];
        d[i].shortfall = demand[i] - share[i];
    }

    // ---- 4. borrowing KVC that a running request releases before the borrower runs out
    std::vector<char> lends(n, 0);
    for (int64_t i = 0; i < n; ++i) {
        if (!d[i].in_batch || d[i].shortfall <= 0) continue;
        const int64_t holds = req[i].allocated + d[i].grant;
        const int64_t occupied = req[i].state == KVCP_WAITING ? req[i].prompt_len : req[i].used;
        const int64_t runs_for = holds - occupied;  // iterations until it exhausts what it holds
        int64_t best = -1, best_left = -1, best_amount = 0;
        for (int64_t j = 0; j < n; ++j) {
            if (j == i || req[j].state != KVCP_RUNNING || !d[j].in_batch || lends[j]) continue;
            const int64_t left = std::max<int64_t>(0, req[j].est_output_len - req[j].generated);
            const int64_t amount = req[j].allocated + d[j].grant;
            if (left > runs_for || amount < d[i].shortfall) continue;
            if (best < 0 || left > best_left || (left == best_left && amount < best_amount)) {
                best = j; best_left = left; best_amount = amount;
            }
        }
        if (best >= 0) {
            lends[best] = 1;
            d[i].lender = best;
        }
    }

    std::copy(d.begin(), d.end(), out);
    if (summary) {
        summary->unallocated_after = avail;
        summary->basic_demand = D;
        summary->excess = excess;
        summary->batch_tokens = batch_tokens;
        summary->n_preempted = n_preempted;
        summary->alloc_case = alloc_case;
    }
    return 0;
}

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
