/*
 * CPU oracle for the MoE circuit-schedule path.  TEST INFRASTRUCTURE ONLY: a plain, slow,
 * single-purpose implementation used to check the GPU library and to time a CPU baseline.
 * It shares no code with the GPU path and must never be called from it.
 *
 * What each function follows (paper = "Birkhoff Decompositions and Photonic Interconnects -
 * Wait! Don't Forget the Compute!"):
 *   oracle_route_histogram   Section 2.1 (dispatch: routed tokens are exchanged to reach their
 *                            experts) and Section 3 (the all-to-all communication matrix
 *                            between ranks): entry (s,q) counts the (token, expert) assignments
 *                            of source rank s whose expert lives on rank q.
 *   oracle_decompose_greedy  Section 3.2: repeatedly extract a maximum-weight perfect matching
 *                            of the residual and remove it, until the residual is zero (or a
 *                            cap is hit).  A matched pair ships its whole residual entry; the
 *                            matching lasts as long as its heaviest pair (Section 3.3,
 *                            Section 4.1 "Execution time").
 *   oracle_decompose_bvn     Section 3.1: A = sum_i lambda_i P_i for a matrix with equal line
 *                            sums.  The paper balances with Sinkhorn-Knopp; here the matrix is
 *                            balanced exactly by adding integer padding (north-west-corner
 *                            fill of the row/column deficits), so the matchings re-sum to
 *                            A + padding bit for bit.
 *   oracle_slice_table       Section 2.2 / 4.1: per matching a receiver hears from exactly one
 *                            source and may start computing as soon as that batch arrived; the
 *                            table gives, per (slice, local expert), the rows that arrive.
 *
 * Tie-break (the paper leaves it open): among equally good permutations the lexicographically
 * smallest (sigma(0), sigma(1), ...) is returned, for both decompositions.
 *
 * Every function here is pinned by tests that do not use this file: brute force over all
 * permutations for n <= 6, scipy's assignment solver for the optimal weight, closed forms,
 * conservation / line-sum invariants, and the matching counts of the paper's Figure 2.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_MAX_N 256

/* ------------------------------------------------------------------------------------------
 * Routing histogram.  ids[N][T][topk]; expert e lives on rank e / (E/N).  Ids outside [0,E)
 * are ignored.  counts[N][E] may be NULL.
 * ------------------------------------------------------------------------------------------ */
int oracle_route_histogram(const int32_t *ids, int N, int T, int topk, int E,
                           int32_t *traffic, int32_t *counts)
{
    if (N <= 0 || E <= 0 || E % N != 0 || T < 0 || topk <= 0) return -1;
    int e_loc = E / N;
    memset(traffic, 0, sizeof(int32_t) * (size_t)N * N);
    if (counts) memset(counts, 0, sizeof(int32_t) * (size_t)N * E);
    for (int s = 0; s < N; ++s)
        for (int t = 0; t < T; ++t)
            for (int j = 0; j < topk; ++j) {
                int32_t e = ids[((size_t)s * T + t) * topk + j];
                if (e < 0 || e >= E) continue;
                traffic[(size_t)s * N + e / e_loc] += 1;
                if (counts) counts[(size_t)s * E + e] += 1;
            }
    return 0;
}

/* ------------------------------------------------------------------------------------------
 * Maximum-weight perfect matching with optimal duals (Kuhn-Munkres, O(n^3), shortest
 * augmenting paths with potentials).  Works on cost = -w.  On return row_to_col is an optimal
 * assignment and (pu[i], pv[j]) satisfy pu[i] + pv[j] >= w[i][j] with equality on every edge
 * of every optimal assignment.
 * ------------------------------------------------------------------------------------------ */
static void max_weight_assignment(const int32_t *w, int n, int *row_to_col, int64_t *pu, int64_t *pv)
{
    /* 1-based arrays in the classical formulation; column 0 is a virtual start column. */
    int64_t u[ORACLE_MAX_N + 1], v[ORACLE_MAX_N + 1], minv[ORACLE_MAX_N + 1];
    int p[ORACLE_MAX_N + 1], way[ORACLE_MAX_N + 1];
    char used[ORACLE_MAX_N + 1];
    const int64_t INF = (int64_t)1 << 60;
    for (int i = 0; i <= n; ++i) { u[i] = 0; v[i] = 0; p[i] = 0; way[i] = 0; }
    for (int i = 1; i <= n; ++i) {
        p[0] = i;
        int j0 = 0;
        for (int j = 0; j <= n; ++j) { minv[j] = INF; used[j] = 0; }
        do {
            used[j0] = 1;
            int i0 = p[j0], j1 = 0;
            int64_t delta = INF;
            for (int j = 1; j <= n; ++j) {
                if (used[j]) continue;
                int64_t cur = -(int64_t)w[(size_t)(i0 - 1) * n + (j - 1)] - u[i0] - v[j];
                if (cur < minv[j]) { minv[j] = cur; way[j] = j0; }
                if (minv[j] < delta) { delta = minv[j]; j1 = j; }
            }
            for (int j = 0; j <= n; ++j) {
                if (used[j]) { u[p[j]] += delta; v[j] -= delta; }
                else minv[j] -= delta;
            }
            j0 = j1;
        } while (p[j0] != 0);
        do {
            int j1 = way[j0];
            p[j0] = p[j1];
            j0 = j1;
        } while (j0);
    }
    for (int j = 1; j <= n; ++j) row_to_col[p[j] - 1] = j - 1;
    /* cost duals satisfy u + v <= -w; negate to get weight duals with pu + pv >= w */
    for (int i = 0; i < n; ++i) { pu[i] = -u[i + 1]; pv[i] = -v[i + 1]; }
}

/* ------------------------------------------------------------------------------------------
 * Lexicographically smallest perfect matching of a bipartite graph given by allowed[i*n+j],
 * starting from some perfect matching row_to_col of that graph.
 * Rows are fixed one after the other.  For row i the allowed columns below its current one
 * that are not held by an already fixed row are tried in ascending order: row i takes column
 * c, the row that held c is evicted and must find another column through an alternating path
 * that only re-routes rows > i and ends in the column row i gave up.  The first success is
 * kept.  A row proven unable to reach the free column stays so for the later candidates of
 * the same row i, because a failed search changes nothing.
 * ------------------------------------------------------------------------------------------ */
typedef struct {
    const unsigned char *allowed;
    int n, fixed_upto, free_col;
    int *row_to_col, *col_to_row;
    char *visited;
} lex_ctx;

static int lex_reroute(lex_ctx *c, int r)
{
    c->visited[r] = 1;
    for (int j = 0; j < c->n; ++j) {
        if (!c->allowed[(size_t)r * c->n + j]) continue;
        if (j == c->free_col) {
            c->row_to_col[r] = j; c->col_to_row[j] = r;
            return 1;
        }
        int r2 = c->col_to_row[j];
        if (r2 <= c->fixed_upto || c->visited[r2]) continue;
        if (lex_reroute(c, r2)) {
            c->row_to_col[r] = j; c->col_to_row[j] = r;
            return 1;
        }
    }
    return 0;
}

static void lex_smallest_matching(const unsigned char *allowed, int n, int *row_to_col)
{
    int col_to_row[ORACLE_MAX_N];
    char visited[ORACLE_MAX_N];
    for (int i = 0; i < n; ++i) col_to_row[row_to_col[i]] = i;
    lex_ctx c = { allowed, n, 0, 0, row_to_col, col_to_row, visited };
    for (int i = 0; i < n; ++i) {
        int cur = row_to_col[i];
        memset(visited, 0, (size_t)n);
        c.fixed_upto = i;
        c.free_col = cur;
        for (int j = 0; j < cur; ++j) {
            if (!allowed[(size_t)i * n + j]) continue;
            int r = col_to_row[j];
            if (r < i) continue;                     /* column belongs to a fixed row */
            if (visited[r]) continue;                /* already shown to be stuck      */
            if (lex_reroute(&c, r)) {
                row_to_col[i] = j; col_to_row[j] = i;
                break;
            }
        }
    }
}

/* FNV-1a, 64 bit, over the byte stream  sigma_t(0..n-1) (one byte each), duration_t (4 bytes,
 * little endian), t = 0..count-1. */
uint64_t oracle_schedule_hash(const uint8_t *perms, const int32_t *durations, int count, int n)
{
    uint64_t h = 14695981039346656037ULL;
    for (int t = 0; t < count; ++t) {
        for (int i = 0; i < n; ++i) { h ^= perms[(size_t)t * n + i]; h *= 1099511628211ULL; }
        uint32_t d = (uint32_t)durations[t];
        for (int b = 0; b < 4; ++b) { h ^= (d >> (8 * b)) & 0xFF; h *= 1099511628211ULL; }
    }
    return h;
}

/* ------------------------------------------------------------------------------------------
 * Greedy max-weight decomposition of one n x n matrix.
 *   perms[kmax][n], durations[kmax]: written for t < returned count; residual[n][n] always.
 * Returns the number of matchings, or -1 on bad arguments.
 * ------------------------------------------------------------------------------------------ */
int oracle_decompose_greedy(const int32_t *A, int n, int kmax, int zero_diag,
                            uint8_t *perms, int32_t *durations, int32_t *residual)
{
    if (n <= 0 || n > ORACLE_MAX_N || kmax < 0) return -1;
    int32_t *R = residual;
    memcpy(R, A, sizeof(int32_t) * (size_t)n * n);
    if (zero_diag) for (int i = 0; i < n; ++i) R[(size_t)i * n + i] = 0;
    unsigned char *tight = (unsigned char *)malloc((size_t)n * n);
    int sigma[ORACLE_MAX_N];
    int64_t pu[ORACLE_MAX_N], pv[ORACLE_MAX_N];
    int count = 0;
    while (count < kmax) {
        int any = 0;
        for (size_t x = 0; x < (size_t)n * n; ++x) if (R[x] != 0) { any = 1; break; }
        if (!any) break;
        max_weight_assignment(R, n, sigma, pu, pv);
        /* the optimal permutations are exactly the perfect matchings of the tight graph */
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < n; ++j)
                tight[(size_t)i * n + j] = (pu[i] + pv[j] == (int64_t)R[(size_t)i * n + j]);
        lex_smallest_matching(tight, n, sigma);
        int32_t dmax = 0;
        for (int i = 0; i < n; ++i) {
            int32_t x = R[(size_t)i * n + sigma[i]];
            if (x > dmax) dmax = x;
            R[(size_t)i * n + sigma[i]] = 0;
            perms[(size_t)count * n + i] = (uint8_t)sigma[i];
        }
        durations[count] = dmax;
        ++count;
    }
    free(tight);
    return count;
}

/* ------------------------------------------------------------------------------------------
 * Integer padding to equal line sums: target = max over all row and column sums; the row and
 * column deficits are filled with the north-west-corner rule.  pad[n][n] receives the padding.
 * ------------------------------------------------------------------------------------------ */
static int32_t pad_to_equal_line_sums(const int32_t *A, int n, int32_t *pad)
{
    int64_t rs[ORACLE_MAX_N], cs[ORACLE_MAX_N], target = 0;
    for (int i = 0; i < n; ++i) { rs[i] = 0; cs[i] = 0; }
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < n; ++j) { rs[i] += A[(size_t)i * n + j]; cs[j] += A[(size_t)i * n + j]; }
    for (int i = 0; i < n; ++i) { if (rs[i] > target) target = rs[i]; if (cs[i] > target) target = cs[i]; }
    for (int i = 0; i < n; ++i) { rs[i] = target - rs[i]; cs[i] = target - cs[i]; }
    memset(pad, 0, sizeof(int32_t) * (size_t)n * n);
    int i = 0, j = 0;
    while (i < n && j < n) {
        if (rs[i] == 0) { ++i; continue; }
        if (cs[j] == 0) { ++j; continue; }
        int64_t dl = rs[i] < cs[j] ? rs[i] : cs[j];
        pad[(size_t)i * n + j] += (int32_t)dl;
        rs[i] -= dl; cs[j] -= dl;
    }
    return (int32_t)target;
}

/* Kuhn's augmenting-path step for the plain (unweighted) matching used to repair the BvN
 * matching after entries reached zero. */
static int kuhn_try(const unsigned char *allowed, int n, int r, int *row_to_col, int *col_to_row, char *seen)
{
    for (int j = 0; j < n; ++j) {
        if (!allowed[(size_t)r * n + j] || seen[j]) continue;
        seen[j] = 1;
        if (col_to_row[j] < 0 || kuhn_try(allowed, n, col_to_row[j], row_to_col, col_to_row, seen)) {
            row_to_col[r] = j; col_to_row[j] = r;
            return 1;
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------------------------
 * Birkhoff-von Neumann decomposition of the padded matrix.
 *   perms, durations (= lambda_t), residual (padded residual, zero when uncapped) as for greedy;
 *   *pad_total = the common line sum; pad_out[n][n] (may be NULL) = the padding that was added.
 * Returns the number of matchings, -1 on bad arguments, -2 if no perfect matching exists in
 * the support (cannot happen for equal line sums; kept as an assertion of the invariant).
 * ------------------------------------------------------------------------------------------ */
int oracle_decompose_bvn(const int32_t *A, int n, int kmax, int zero_diag,
                         uint8_t *perms, int32_t *durations, int32_t *residual,
                         int32_t *pad_total, int32_t *pad_out)
{
    if (n <= 0 || n > ORACLE_MAX_N || kmax < 0) return -1;
    int32_t *R = residual;
    memcpy(R, A, sizeof(int32_t) * (size_t)n * n);
    if (zero_diag) for (int i = 0; i < n; ++i) R[(size_t)i * n + i] = 0;
    int32_t *pad = (int32_t *)malloc(sizeof(int32_t) * (size_t)n * n);
    *pad_total = pad_to_equal_line_sums(R, n, pad);
    for (size_t x = 0; x < (size_t)n * n; ++x) R[x] += pad[x];
    if (pad_out) memcpy(pad_out, pad, sizeof(int32_t) * (size_t)n * n);
    free(pad);

    unsigned char *support = (unsigned char *)malloc((size_t)n * n);
    int row_to_col[ORACLE_MAX_N], col_to_row[ORACLE_MAX_N];
    char seen[ORACLE_MAX_N];
    for (int i = 0; i < n; ++i) { row_to_col[i] = -1; col_to_row[i] = -1; }
    int count = 0, status = 0;
    while (count < kmax) {
        int any = 0;
        for (size_t x = 0; x < (size_t)n * n; ++x) { support[x] = R[x] > 0; any |= support[x]; }
        if (!any) break;
        /* (re)match every row that has no valid edge */
        for (int i = 0; i < n && status == 0; ++i) {
            if (row_to_col[i] >= 0) continue;
            memset(seen, 0, (size_t)n);
            if (!kuhn_try(support, n, i, row_to_col, col_to_row, seen)) status = -2;
        }
        if (status) break;
        lex_smallest_matching(support, n, row_to_col);
        for (int i = 0; i < n; ++i) col_to_row[row_to_col[i]] = i;
        int32_t lambda = R[row_to_col[0]];
        for (int i = 1; i < n; ++i) {
            int32_t x = R[(size_t)i * n + row_to_col[i]];
            if (x < lambda) lambda = x;
        }
        for (int i = 0; i < n; ++i) {
            perms[(size_t)count * n + i] = (uint8_t)row_to_col[i];
            R[(size_t)i * n + row_to_col[i]] -= lambda;
        }
        durations[count] = lambda;
        ++count;
        for (int i = 0; i < n; ++i)
            if (R[(size_t)i * n + row_to_col[i]] == 0) { col_to_row[row_to_col[i]] = -1; row_to_col[i] = -1; }
    }
    free(support);
    return status ? status : count;
}

/* ------------------------------------------------------------------------------------------
 * Sinkhorn-Knopp scaling followed by Birkhoff-von Neumann on the scaled matrix (Section 3.1:
 * "a preprocessing step such as Sinkhorn-Knopp normalization is required before decomposition
 * can be applied").  Double precision throughout.
 *   X <- A (diagonal zeroed on request); `iters` times: every row with a positive sum is divided
 *   by its sum, then every column with a positive sum by its sum (sums taken left to right / top
 *   to bottom).  *deviation = max_i |row sum - 1| afterwards.
 *   Then while fewer than kmax matchings: the support is {X > eps}; stop when it is empty or
 *   holds no perfect matching (the scaling is approximate, so the last crumbs need not be
 *   decomposable); sigma <- lexicographically smallest perfect matching of the support;
 *   lambda <- min_i X[i][sigma(i)]; X[i][sigma(i)] -= lambda.
 * scaled_out (may be NULL) receives X after the scaling, residual what is left at the end.
 * The paper fixes neither the number of sweeps nor a tolerance: both are arguments.
 * ------------------------------------------------------------------------------------------ */
int oracle_sinkhorn_bvn(const int32_t *A, int n, int kmax, int zero_diag, int iters, double eps,
                        uint8_t *perms, double *coeffs, double *scaled_out, double *residual,
                        double *deviation)
{
    if (n <= 0 || n > ORACLE_MAX_N || kmax < 0 || iters < 0 || !(eps >= 0.0)) return -1;
    double *X = residual;
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < n; ++j)
            X[(size_t)i * n + j] = (zero_diag && i == j) ? 0.0 : (double)A[(size_t)i * n + j];
    for (int it = 0; it < iters; ++it) {
        for (int i = 0; i < n; ++i) {
            double sum = 0.0;
            for (int j = 0; j < n; ++j) sum += X[(size_t)i * n + j];
            if (sum > 0.0) for (int j = 0; j < n; ++j) X[(size_t)i * n + j] = X[(size_t)i * n + j] / sum;
        }
        for (int j = 0; j < n; ++j) {
            double sum = 0.0;
            for (int i = 0; i < n; ++i) sum += X[(size_t)i * n + j];
            if (sum > 0.0) for (int i = 0; i < n; ++i) X[(size_t)i * n + j] = X[(size_t)i * n + j] / sum;
        }
    }
    double dev = 0.0;
    for (int i = 0; i < n; ++i) {
        double sum = 0.0;
        for (int j = 0; j < n; ++j) sum += X[(size_t)i * n + j];
        double d = sum > 1.0 ? sum - 1.0 : 1.0 - sum;
        if (d > dev) dev = d;
    }
    if (deviation) *deviation = dev;
    if (scaled_out) memcpy(scaled_out, X, sizeof(double) * (size_t)n * n);

    unsigned char *support = (unsigned char *)malloc((size_t)n * n);
    int row_to_col[ORACLE_MAX_N], col_to_row[ORACLE_MAX_N];
    char seen[ORACLE_MAX_N];
    for (int i = 0; i < n; ++i) { row_to_col[i] = -1; col_to_row[i] = -1; }
    int count = 0, stuck = 0;
    while (count < kmax && !stuck) {
        int any = 0;
        for (size_t x = 0; x < (size_t)n * n; ++x) { support[x] = X[x] > eps; any |= support[x]; }
        if (!any) break;
        for (int i = 0; i < n && !stuck; ++i) {
            if (row_to_col[i] >= 0) continue;
            memset(seen, 0, (size_t)n);
            if (!kuhn_try(support, n, i, row_to_col, col_to_row, seen)) stuck = 1;
        }
        if (stuck) break;
        lex_smallest_matching(support, n, row_to_col);
        for (int i = 0; i < n; ++i) col_to_row[row_to_col[i]] = i;
        double lambda = X[row_to_col[0]];
        for (int i = 1; i < n; ++i) {
            double x = X[(size_t)i * n + row_to_col[i]];
            if (x < lambda) lambda = x;
        }
        for (int i = 0; i < n; ++i) {
            perms[(size_t)count * n + i] = (uint8_t)row_to_col[i];
            X[(size_t)i * n + row_to_col[i]] = X[(size_t)i * n + row_to_col[i]] - lambda;
        }
        coeffs[count] = lambda;
        ++count;
        for (int i = 0; i < n; ++i)
            if (!(X[(size_t)i * n + row_to_col[i]] > eps)) { col_to_row[row_to_col[i]] = -1; row_to_col[i] = -1; }
    }
    free(support);
    return count;
}

/* ------------------------------------------------------------------------------------------
 * Batched drivers (independent matrices), optionally spread over OpenMP threads.
 * perms may be NULL (only counts / durations / hashes wanted); scratch is then local.
 * ------------------------------------------------------------------------------------------ */
int oracle_decompose_batch(int which /*0 greedy, 1 bvn*/, const int32_t *mats, int B, int n, int kmax,
                           int zero_diag, uint8_t *perms, int32_t *durations, int32_t *counts,
                           int32_t *residual, int32_t *pad_total, uint64_t *hashes, int nthreads)
{
    int bad = 0;
    if (nthreads < 1) nthreads = 1;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
    for (int b = 0; b < B; ++b) {
        uint8_t *pp = perms ? perms + (size_t)b * kmax * n : (uint8_t *)malloc((size_t)kmax * n + 1);
        int32_t *dd = durations ? durations + (size_t)b * kmax : (int32_t *)malloc(sizeof(int32_t) * ((size_t)kmax + 1));
        int32_t *rr = residual ? residual + (size_t)b * n * n : (int32_t *)malloc(sizeof(int32_t) * (size_t)n * n);
        int32_t pt = 0;
        int c = which == 0
            ? oracle_decompose_greedy(mats + (size_t)b * n * n, n, kmax, zero_diag, pp, dd, rr)
            : oracle_decompose_bvn(mats + (size_t)b * n * n, n, kmax, zero_diag, pp, dd, rr, &pt, NULL);
        if (c < 0) {
#pragma omp atomic write
            bad = 1;
            c = 0;
        }
        counts[b] = c;
        if (pad_total) pad_total[b] = pt;
        if (hashes) hashes[b] = oracle_schedule_hash(pp, dd, c, n);
        if (!perms) free(pp);
        if (!durations) free(dd);
        if (!residual) free(rr);
    }
    return bad ? -1 : 0;
}

/* ------------------------------------------------------------------------------------------
 * Slice table of receiving rank r.
 *   traffic[N][N]       histogram output (diagonal included; local pairs never use a circuit).
 *   perms/durations     schedule of `count` matchings, stored with stride kmax.
 * Slices: 0 = local pairs (source r); 1 + t = what matching t delivers, t < kmax (empty for
 * t >= count); kmax + 1 = whatever the schedule did not ship, by source, then arrival order.
 * On matching t the pair (s, sigma_t(s)) ships min(remaining, duration_t) assignments, taken
 * first-in-first-out from source s's (token, slot) sequence restricted to experts on r.
 * Inside a slice rows are stably grouped by local expert.
 *   offsets[(kmax+2)*E_loc + 1]  row boundaries of the (slice, expert) groups.
 *   row_src[M] (may be NULL)     for every grouped row the flat index (s*T + t)*topk + j of
 *                                the assignment it carries.
 * Returns M (rows received by r), or -1.
 * ------------------------------------------------------------------------------------------ */
int oracle_slice_table(const int32_t *ids, int N, int T, int topk, int E, int r,
                       const int32_t *traffic, const uint8_t *perms, const int32_t *durations,
                       int count, int kmax, int32_t *offsets, int32_t *row_src)
{
    if (N <= 0 || E % N != 0 || r < 0 || r >= N || count < 0 || count > kmax) return -1;
    int e_loc = E / N, S = kmax + 2;
    size_t per_src = (size_t)T * topk;
    /* slice index of every assignment destined to r (or -1) */
    int32_t *slice_of = (int32_t *)malloc(sizeof(int32_t) * (size_t)N * per_src);
    for (int s = 0; s < N; ++s) {
        /* window boundaries in source s's arrival sequence */
        int64_t *cum = (int64_t *)malloc(sizeof(int64_t) * ((size_t)count + 1));
        int64_t remaining = (s == r) ? 0 : traffic[(size_t)s * N + r], shipped = 0;
        for (int t = 0; t < count; ++t) {
            if (s != r && perms[(size_t)t * N + s] == r) {
                int64_t ship = remaining < durations[t] ? remaining : durations[t];
                remaining -= ship; shipped += ship;
            }
            cum[t] = shipped;                        /* assignments shipped up to and incl. t */
        }
        int64_t q = 0;                               /* position in the filtered sequence */
        for (size_t x = 0; x < per_src; ++x) {
            int32_t e = ids[(size_t)s * per_src + x];
            int32_t sl = -1;
            if (e >= 0 && e < E && e / e_loc == r) {
                if (s == r) sl = 0;
                else {
                    int t = 0;
                    while (t < count && cum[t] <= q) ++t;
                    sl = (t < count) ? 1 + t : kmax + 1;
                }
                ++q;
            }
            slice_of[(size_t)s * per_src + x] = sl;
        }
        free(cum);
    }
    size_t G = (size_t)S * e_loc;
    int64_t *size = (int64_t *)calloc(G, sizeof(int64_t));
    for (size_t x = 0; x < (size_t)N * per_src; ++x)
        if (slice_of[x] >= 0) size[(size_t)slice_of[x] * e_loc + (ids[x] % e_loc)] += 1;
    offsets[0] = 0;
    for (size_t g = 0; g < G; ++g) offsets[g + 1] = offsets[g] + (int32_t)size[g];
    if (row_src) {
        int64_t *fill = (int64_t *)calloc(G, sizeof(int64_t));
        for (size_t x = 0; x < (size_t)N * per_src; ++x)      /* source-major, then arrival order */
            if (slice_of[x] >= 0) {
                size_t g = (size_t)slice_of[x] * e_loc + (ids[x] % e_loc);
                row_src[offsets[g] + fill[g]++] = (int32_t)x;
            }
        free(fill);
    }
    int M = offsets[G];
    free(size);
    free(slice_of);
    return M;
}
