// Cluster-level KV placement (Section 5.3): per-layer performance model (Eq. 5, Eq. 6), instance and cluster
// throughput (Eq. 7) and the greedy debtor / creditor scheduler (Algorithm 1).  Host code, fp64.
//
// Each instance is reduced once to a handful of totals, so an estimate costs O(1).  For a fixed number of admitted
// requests the pair's estimate beta'/(n (a - k x)) + beta_c/(n (b + k x)) is convex in k, so its maximum over a
// range of k lies at an end of one of the stretches between two admissions: only those ends are evaluated
// (at most 2 min(waiting, table room) + 2 candidates instead of Block_max).
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <vector>

#include "../../include/distattn_placement.h"

namespace {

struct Totals {
    int32_t beta = 0;        // requests, admitted ones included
    int64_t own_tokens = 0;  // sum of S^r, admitted ones included
    int64_t own_blocks = 0;  // blocks of those requests, wherever they are
    int64_t remote = 0;      // of them, held by creditors
    int64_t remote_tokens = 0;  // tokens in those blocks (a remote last block may be partly filled)
    int64_t hosted = 0;      // blocks held for others
    int64_t capacity = 0;
    int32_t waiting = 0;
    int32_t admit_blocks = 0;
    int64_t used() const { return own_blocks - remote + hosted; }
    double utilisation() const { return (double)used() / (double)capacity; }
};

bool valid_model(const da_perf_model *m)
{
    if (!m || !m->t_natn || m->t_natn_len < 1 || m->num_layers < 1 || m->block_tokens < 1) return false;
    if (!(m->attn_tokens_per_s > 0.0)) return false;  // also rejects NaN
    for (int32_t b = 0; b < m->t_natn_len; ++b)
        if (!std::isfinite(m->t_natn[b]) || m->t_natn[b] < 0.0) return false;
    return true;
}

bool reduce(const da_perf_model &m, const da_instance &in, Totals *out)
{
    Totals t;
    if (in.num_requests < 0 || in.num_requests > m.t_natn_len - 1) return false;
    if (in.num_requests > 0 && !in.req_tokens) return false;
    if (in.hosted_blocks < 0 || in.capacity_blocks < 1 || in.waiting < 0 || in.admit_blocks < 0) return false;
    for (int32_t r = 0; r < in.num_requests; ++r) {
        const int64_t s = in.req_tokens[r];
        if (s < 1) return false;
        const int64_t nb = (s + m.block_tokens - 1) / m.block_tokens;
        const int64_t rb = in.req_remote_blocks ? in.req_remote_blocks[r] : 0;
        if (rb < 0 || rb > nb) return false;
        t.own_tokens += s;
        t.own_blocks += nb;
        t.remote += rb;
        t.remote_tokens += std::min<int64_t>(rb * m.block_tokens, s);
    }
    t.beta = in.num_requests;
    t.hosted = in.hosted_blocks;
    t.capacity = in.capacity_blocks;
    t.waiting = in.waiting;
    t.admit_blocks = in.admit_blocks;
    *out = t;
    return true;
}

// requests admitted from the queue once k more blocks have left (beta' - beta of Eq. 6)
int32_t admitted_after(const da_perf_model &m, const Totals &t, int64_t k)
{
    if (t.admit_blocks <= 0 || t.waiting <= 0) return 0;
    const int64_t free_blocks = t.capacity - t.used() + k;
    if (free_blocks <= 0) return 0;
    int64_t a = std::min<int64_t>(t.waiting, free_blocks / t.admit_blocks);
    a = std::min<int64_t>(a, (int64_t)m.t_natn_len - 1 - t.beta);
    return (int32_t)std::max<int64_t>(a, 0);
}

// TPS with `out` more blocks placed remotely, `in` more blocks hosted and `a` more requests admitted
double tps_of(const da_perf_model &m, const Totals &t, int64_t out, int64_t in, int32_t a)
{
    const int32_t beta = t.beta + a;
    if (beta == 0) return 0.0;
    const int64_t T = m.block_tokens;
    const int64_t tokens = t.own_tokens + (int64_t)a * t.admit_blocks * T - t.remote_tokens - out * T + (t.hosted + in) * T;
    const double layer = m.t_natn[beta] + (double)tokens / m.attn_tokens_per_s;
    return (double)beta / ((double)m.num_layers * layer);
}

double pair_estimate(const da_perf_model &m, const Totals &d, const Totals &c, int64_t k)
{
    return tps_of(m, d, k, 0, admitted_after(m, d, k)) + tps_of(m, c, 0, k, 0);
}

// smallest k in [0, kmax] with the largest estimate
int64_t best_blocks(const da_perf_model &m, const Totals &d, const Totals &c, int64_t kmax)
{
    int64_t best_k = 0;
    double best = pair_estimate(m, d, c, 0);
    auto consider = [&](int64_t k) {
        if (k <= 0 || k > kmax) return;
        const double p = pair_estimate(m, d, c, k);
        if (p > best) {
            best = p;
            best_k = k;
        }
    };
    const int32_t a_first = admitted_after(m, d, 0);
    const int32_t a_last = admitted_after(m, d, kmax);
    const int64_t free0 = d.capacity - d.used();
    for (int32_t j = a_first + 1; j <= a_last; ++j) {
        const int64_t kj = (int64_t)j * d.admit_blocks - free0;  // first k at which the j-th request fits
        consider(kj - 1);
        consider(kj);
    }
    consider(kmax);
    return best_k;
}

}  // namespace

extern "C" {

da_status da_model_instance_tps(const da_perf_model *model, const da_instance *instance, double *tps)
{
    Totals t;
    if (!valid_model(model) || !instance || !tps || !reduce(*model, *instance, &t)) return DA_ERR_INVALID_ARG;
    *tps = tps_of(*model, t, 0, 0, 0);
    return DA_OK;
}

da_status da_model_cluster_tps(const da_perf_model *model, const da_instance *instances, int32_t num_instances,
                               double *tps)
{
    if (!valid_model(model) || !tps || num_instances < 0 || (num_instances > 0 && !instances)) return DA_ERR_INVALID_ARG;
    double sum = 0.0;
    for (int32_t i = 0; i < num_instances; ++i) {
        Totals t;
        if (!reduce(*model, instances[i], &t)) return DA_ERR_INVALID_ARG;
        sum += tps_of(*model, t, 0, 0, 0);
    }
    *tps = sum;
    return DA_OK;
}

da_status da_model_pair_estimate(const da_perf_model *model, const da_instance *debtor, const da_instance *creditor,
                                 int32_t k, double *tps)
{
    Totals d, c;
    if (!valid_model(model) || !debtor || !creditor || !tps || k < 0) return DA_ERR_INVALID_ARG;
    if (!reduce(*model, *debtor, &d) || !reduce(*model, *creditor, &c)) return DA_ERR_INVALID_ARG;
    *tps = pair_estimate(*model, d, c, k);
    return DA_OK;
}

da_status da_placement_schedule(const da_perf_model *model, const da_instance *instances, int32_t num_instances,
                                int32_t beta_thres, double u_thres, da_move *moves, int32_t max_moves,
                                int32_t *num_moves, double *tps_before, double *tps_after)
{
    if (!valid_model(model) || !num_moves || num_instances < 0 || (num_instances > 0 && !instances) || max_moves < 0 ||
        (max_moves > 0 && !moves) || std::isnan(u_thres))
        return DA_ERR_INVALID_ARG;
    const da_perf_model &m = *model;
    std::vector<Totals> st((size_t)num_instances);
    for (int32_t i = 0; i < num_instances; ++i)
        if (!reduce(m, instances[i], &st[i])) return DA_ERR_INVALID_ARG;
    auto cluster = [&]() {
        double s = 0.0;
        for (const Totals &t : st) s += tps_of(m, t, 0, 0, 0);
        return s;
    };
    if (tps_before) *tps_before = cluster();

    // roles, fixed for the call
    std::vector<int32_t> debtors, creditors;
    for (int32_t i = 0; i < num_instances; ++i) {
        const bool lender = st[i].utilisation() <= u_thres && st[i].remote == 0;
        if (lender)
            creditors.push_back(i);
        else if (st[i].beta <= beta_thres && st[i].beta > 0 && st[i].hosted == 0)
            debtors.push_back(i);
    }
    std::stable_sort(debtors.begin(), debtors.end(), [&](int32_t a, int32_t b) { return st[a].beta < st[b].beta; });

    int32_t count = 0;
    std::vector<uint8_t> tried((size_t)num_instances);
    for (int32_t d : debtors) {
        const da_instance &in = instances[d];
        int32_t r = 0;
        for (int32_t x = 1; x < in.num_requests; ++x)
            if (in.req_tokens[x] > in.req_tokens[r]) r = x;
        int64_t block_max = (in.req_tokens[r] + m.block_tokens - 1) / m.block_tokens -
                            (in.req_remote_blocks ? in.req_remote_blocks[r] : 0);
        std::fill(tried.begin(), tried.end(), 0);
        for (;;) {
            int32_t c = -1;
            double c_util = 0.0;
            for (int32_t x : creditors) {
                if (tried[x]) continue;
                const double u = st[x].utilisation();
                if (c < 0 || u < c_util) {
                    c = x;
                    c_util = u;
                }
            }
            if (c < 0) break;
            tried[c] = 1;
            const int64_t kmax = std::min<int64_t>(block_max - 1, st[c].capacity - st[c].used());
            const int64_t k = kmax > 0 ? best_blocks(m, st[d], st[c], kmax) : 0;
            if (k <= 0) break;
            const int32_t a = admitted_after(m, st[d], k);
            st[d].remote += k;
            st[d].remote_tokens += k * m.block_tokens;
            st[d].beta += a;
            st[d].waiting -= a;
            st[d].own_tokens += (int64_t)a * st[d].admit_blocks * m.block_tokens;
            st[d].own_blocks += (int64_t)a * st[d].admit_blocks;
            st[c].hosted += k;
            if (count < max_moves) moves[count] = da_move{d, r, c, (int32_t)k};
            ++count;
            block_max -= k;
        }
    }
    *num_moves = count;
    if (tps_after) *tps_after = cluster();
    return count > max_moves ? DA_ERR_WORKSPACE : DA_OK;
}

}  // extern "C"
