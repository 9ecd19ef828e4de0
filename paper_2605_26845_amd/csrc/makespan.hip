// moe_makespan_model / moe_order_matchings: analytic completion time of one MoE layer under a
// circuit schedule (Section 5, Setup: "Execution time") and Johnson's ordering of the matchings
// (Section 4: ordering as a flow-shop problem).  Host code only: the inputs are a handful of
// N x N integers and K permutations; nothing here touches the GPU.
#include "common.hpp"
#include <algorithm>
#include <vector>

namespace {

struct Cost {
    const moe_cost_model& m;
    double comm(long long rows) const { return m.reconf_s + (double)rows * m.bytes_per_row / m.bandwidth; }
    double wire(long long rows) const { return (double)rows * m.bytes_per_row / m.bandwidth; }
    double compute(long long rows) const {
        if (rows <= 0) return 0.0;
        const double r = (double)rows;
        if (m.kind == MOE_COST_LINEAR) return m.fixed_s + m.per_row_s * r;
        const double* x = m.table_rows;
        const double* y = m.table_seconds;
        const int L = m.table_len;
        if (r <= x[0]) return y[0];
        int hi = (int)(std::lower_bound(x, x + L, r) - x);          // first point with x >= r
        if (hi >= L) hi = L - 1;                                      // beyond the table: last segment continued
        const int lo = hi - 1;
        return y[lo] + (r - x[lo]) * (y[hi] - y[lo]) / (x[hi] - x[lo]);
    }
};

bool valid_cost(const moe_cost_model* c) {
    if (!c || !(c->bandwidth > 0.0) || c->bytes_per_row < 0.0 || c->reconf_s < 0.0) return false;
    if (c->kind == MOE_COST_LINEAR) return c->fixed_s >= 0.0 && c->per_row_s >= 0.0;
    if (c->kind != MOE_COST_TABLE || c->table_len < 2 || !c->table_rows || !c->table_seconds) return false;
    for (int i = 1; i < c->table_len; ++i)
        if (!(c->table_rows[i] > c->table_rows[i - 1])) return false;
    return true;
}

// received[t * N + j] = rows rank j receives in matching t (original order); rest = what is left of the matrix
void play_schedule(const int32_t* traffic, int N, const uint8_t* perms, const int32_t* durations, int K,
                   std::vector<long long>& received, std::vector<long long>& rest) {
    rest.assign((size_t)N * N, 0);
    for (int i = 0; i < N; ++i)
        for (int j = 0; j < N; ++j)
            if (i != j) rest[(size_t)i * N + j] = traffic[(size_t)i * N + j];
    received.assign((size_t)K * N, 0);
    for (int t = 0; t < K; ++t)
        for (int i = 0; i < N; ++i) {
            const int j = perms[(size_t)t * N + i];
            if (j == i || j >= N) continue;
            long long& cell = rest[(size_t)i * N + j];
            const long long s = std::min<long long>(cell, durations[t]);
            cell -= s;
            received[(size_t)t * N + j] = s;
        }
}

moe_status check_common(const int32_t* traffic, int N, const uint8_t* perms, const int32_t* durations, int K,
                        const moe_cost_model* cost) {
    if (!traffic || N < 1 || K < 0 || (K > 0 && (!perms || !durations)) || !valid_cost(cost)) return MOE_ERR_INVALID_ARG;
    if (N > 256) return MOE_ERR_UNSUPPORTED_SHAPE;
    return MOE_OK;
}

}  // namespace

extern "C" moe_status moe_makespan_model(const int32_t* traffic, int N, const uint8_t* perms, const int32_t* durations,
                                         int K, const int32_t* order, const moe_cost_model* cost, double* out) {
    moe_status st = check_common(traffic, N, perms, durations, K, cost);
    if (st != MOE_OK) return st;
    if (!out) return MOE_ERR_INVALID_ARG;
    std::vector<int> seq(K);
    {
        std::vector<char> seen(K, 0);
        for (int t = 0; t < K; ++t) {
            const int o = order ? order[t] : t;
            if (o < 0 || o >= K || seen[o]) return MOE_ERR_INVALID_ARG;
            seen[o] = 1;
            seq[t] = o;
        }
    }
    const Cost c{*cost};
    std::vector<long long> received, rest;
    play_schedule(traffic, N, perms, durations, K, received, rest);

    // network phases: the matchings in play order, then one round for what is left
    struct Phase { double net; std::vector<double> work; std::vector<char> has; };
    std::vector<Phase> phases;
    for (int t = 0; t < K; ++t) {
        Phase p{c.comm(durations[seq[t]]), std::vector<double>(N), std::vector<char>(N)};
        for (int j = 0; j < N; ++j) {
            const long long rows = received[(size_t)seq[t] * N + j];
            p.work[j] = c.compute(rows);
            p.has[j] = rows > 0;
        }
        phases.push_back(std::move(p));
    }
    {
        std::vector<long long> col(N, 0), row(N, 0);
        for (int i = 0; i < N; ++i)
            for (int j = 0; j < N; ++j) { col[j] += rest[(size_t)i * N + j]; row[i] += rest[(size_t)i * N + j]; }
        const long long line = std::max(*std::max_element(col.begin(), col.end()), *std::max_element(row.begin(), row.end()));
        if (line > 0) {
            Phase p{c.comm(line), std::vector<double>(N), std::vector<char>(N)};
            for (int j = 0; j < N; ++j) { p.work[j] = c.compute(col[j]); p.has[j] = col[j] > 0; }
            phases.push_back(std::move(p));
        }
    }
    std::vector<double> local(N);
    for (int j = 0; j < N; ++j) local[j] = c.compute(traffic[(size_t)j * N + j]);
    const double local_max = *std::max_element(local.begin(), local.end());

    // [0] strictly sequential
    double t_seq = local_max, net_sum = 0.0, work_sum = local_max;
    for (const Phase& p : phases) {
        const double w = *std::max_element(p.work.begin(), p.work.end());
        t_seq += 2.0 * p.net + w;
        net_sum += p.net;
        work_sum += w;
    }
    // [1] overlapped: dispatches back to back; each rank works through its slices as they arrive; combines follow
    std::vector<double> busy_until = local;
    std::vector<double> slice_done(phases.size());
    double clock = 0.0;
    for (size_t k = 0; k < phases.size(); ++k) {
        clock += phases[k].net;                                   // dispatch k has arrived
        double fin = clock;
        for (int j = 0; j < N; ++j)
            if (phases[k].has[j]) {
                busy_until[j] = std::max(busy_until[j], clock) + phases[k].work[j];
                fin = std::max(fin, busy_until[j]);
            }
        slice_done[k] = fin;
    }
    for (size_t k = 0; k < phases.size(); ++k) clock = std::max(clock, slice_done[k]) + phases[k].net;
    double t_ovl = clock;
    for (int j = 0; j < N; ++j) t_ovl = std::max(t_ovl, busy_until[j]);
    // [2] idealised congestion-free all-to-all
    long long tstar = 0;
    double biggest = 0.0;
    for (int j = 0; j < N; ++j) {
        long long col = 0, row = 0, all = 0;
        for (int i = 0; i < N; ++i) {
            all += traffic[(size_t)i * N + j];
            if (i != j) { col += traffic[(size_t)i * N + j]; row += traffic[(size_t)j * N + i]; }
        }
        tstar = std::max(tstar, std::max(col, row));
        biggest = std::max(biggest, c.compute(all));
    }
    out[0] = t_seq;
    out[1] = t_ovl;
    out[2] = 2.0 * c.wire(tstar) + biggest;
    out[3] = net_sum;
    out[4] = work_sum;
    return MOE_OK;
}

extern "C" moe_status moe_order_matchings(const int32_t* traffic, int N, const uint8_t* perms, const int32_t* durations,
                                          int K, const moe_cost_model* cost, int32_t* order_out) {
    moe_status st = check_common(traffic, N, perms, durations, K, cost);
    if (st != MOE_OK) return st;
    if (K > 0 && !order_out) return MOE_ERR_INVALID_ARG;
    const Cost c{*cost};
    std::vector<long long> received, rest;
    play_schedule(traffic, N, perms, durations, K, received, rest);
    struct Job { double a, b; int t; };
    std::vector<Job> early, late;                                  // Johnson: a <= b first by a ascending, then the rest by b descending
    for (int t = 0; t < K; ++t) {
        double b = 0.0;
        for (int j = 0; j < N; ++j) b = std::max(b, c.compute(received[(size_t)t * N + j]));
        const Job job{c.comm(durations[t]), b, t};
        (job.a <= job.b ? early : late).push_back(job);
    }
    std::stable_sort(early.begin(), early.end(), [](const Job& x, const Job& y) { return x.a < y.a; });
    std::stable_sort(late.begin(), late.end(), [](const Job& x, const Job& y) { return x.b > y.b; });
    int k = 0;
    for (const Job& j : early) order_out[k++] = j.t;
    for (const Job& j : late) order_out[k++] = j.t;
    return MOE_OK;
}
