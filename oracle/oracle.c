/*
 * CPU checker for the matching-based scheduling round (test infrastructure).
 *
 * This file is the plain, slow statement of what one scheduling round
 * computes (paper: Section "Matching-based scheduling", Algorithm "Scheduling
 * algorithm"): an edge weight for every online x offline pair from the speed
 * predictor, then a maximum-weight bipartite matching over those edges.
 * It exists only so that tests, the smoke check and the benchmark's CPU
 * baseline have something independent to compare the GPU library against;
 * it shares no code with that library and the library never calls it.
 *
 * Everything is straight loops over the definitions: no blocking, no
 * vector intrinsics, no restructured arithmetic.  OpenMP is used only to
 * hand independent rows to different threads.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_INFEASIBLE INT32_MIN

/* ------------------------------------------------------------------------
 * Edge weights: the speed predictor evaluated on one pair.
 *
 * The predictor is an MLP over the profiled features of both workloads
 * (Section "Matching-based scheduling": features of the online and the
 * offline workload are the input, the normalised shared throughput of the
 * offline workload is the output; Section "Implementation": four layers of
 * units with two hidden layers).  Input x = [online features ; offline
 * features] in the argument order of CalcNormTput(u, v, sm).  The SM share
 * sm = DynamicSM(u, v) comes in one of two readings.  sm_on < 0: it is a
 * function of the online workload alone (Section "Dynamic SM allocation":
 * complementary to the online workload's SM activity) and therefore one of
 * its features.  sm_on >= 0: it depends on both workloads - the offline
 * workload gets the complement of the online workload's SM activity (online
 * feature sm_on) but no more than it can use (offline feature sm_off),
 *     sm = min(1 - x_u[sm_on], x_v[sm_off])   (float32 subtraction and minimum)
 * - and is a third input: x = [online ; offline ; sm], W1 has 2F + 1 columns.
 * Hidden activations are ReLU, the output is squashed by a logistic function
 * so that it reads as a fraction in (0,1).
 *
 * sigma_out (optional) receives the score before quantisation; w_out
 * (optional) receives rint(sigma * scale) as int32, or ORC_INFEASIBLE when
 * the two memory fractions (feature `mem_feature` of each side) add up, in
 * one float32 addition, to more than mem_limit.
 *
 * wide != 0: all sums and the exponential in double, one rounding of sigma
 *            to float at the end (the order-independent reference).
 * wide == 0: the same loops entirely in float (shows float32's own noise).
 * ---------------------------------------------------------------------- */
static void score_row_wide(const float *xu, const float *x_off, int m, int F, int H, int sm_on, int sm_off,
                           const float *W1, const float *b1, const float *W2, const float *b2,
                           const float *W3, const float *b3, float *sig_row)
{
    double *h1 = (double *)malloc(sizeof(double) * (size_t)H);
    double *h2 = (double *)malloc(sizeof(double) * (size_t)H);
    const int ld1 = 2 * F + (sm_on >= 0 ? 1 : 0);
    for (int j = 0; j < m; ++j) {
        const float *xv = x_off + (size_t)j * F;
        const float sm = sm_on >= 0 ? fminf(1.0f - xu[sm_on], xv[sm_off]) : 0.0f;
        for (int k = 0; k < H; ++k) {
            double s = (double)b1[k];
            const float *w = W1 + (size_t)k * (size_t)ld1;
            for (int t = 0; t < F; ++t) s += (double)w[t] * (double)xu[t];
            for (int t = 0; t < F; ++t) s += (double)w[F + t] * (double)xv[t];
            if (sm_on >= 0) s += (double)w[2 * F] * (double)sm;
            h1[k] = s > 0.0 ? s : 0.0;
        }
        for (int k = 0; k < H; ++k) {
            double s = (double)b2[k];
            const float *w = W2 + (size_t)k * H;
            for (int t = 0; t < H; ++t) s += (double)w[t] * h1[t];
            h2[k] = s > 0.0 ? s : 0.0;
        }
        double z = (double)b3[0];
        for (int t = 0; t < H; ++t) z += (double)W3[t] * h2[t];
        sig_row[j] = (float)(1.0 / (1.0 + exp(-z)));
    }
    free(h1);
    free(h2);
}

static void score_row_narrow(const float *xu, const float *x_off, int m, int F, int H, int sm_on, int sm_off,
                             const float *W1, const float *b1, const float *W2, const float *b2,
                             const float *W3, const float *b3, float *sig_row)
{
    float *h1 = (float *)malloc(sizeof(float) * (size_t)H);
    float *h2 = (float *)malloc(sizeof(float) * (size_t)H);
    const int ld1 = 2 * F + (sm_on >= 0 ? 1 : 0);
    for (int j = 0; j < m; ++j) {
        const float *xv = x_off + (size_t)j * F;
        const float sm = sm_on >= 0 ? fminf(1.0f - xu[sm_on], xv[sm_off]) : 0.0f;
        for (int k = 0; k < H; ++k) {
            float s = b1[k];
            const float *w = W1 + (size_t)k * (size_t)ld1;
            for (int t = 0; t < F; ++t) s += w[t] * xu[t];
            for (int t = 0; t < F; ++t) s += w[F + t] * xv[t];
            if (sm_on >= 0) s += w[2 * F] * sm;
            h1[k] = s > 0.0f ? s : 0.0f;
        }
        for (int k = 0; k < H; ++k) {
            float s = b2[k];
            const float *w = W2 + (size_t)k * H;
            for (int t = 0; t < H; ++t) s += w[t] * h1[t];
            h2[k] = s > 0.0f ? s : 0.0f;
        }
        float z = b3[0];
        for (int t = 0; t < H; ++t) z += W3[t] * h2[t];
        sig_row[j] = 1.0f / (1.0f + expf(-z));
    }
    free(h1);
    free(h2);
}

int orc_score_pairs(const float *x_on, int n, const float *x_off, int m, int F, int H,
                    const float *W1, const float *b1, const float *W2, const float *b2,
                    const float *W3, const float *b3, float scale, int mem_feature,
                    float mem_limit, int sm_on, int sm_off, int wide, int threads, float *sigma_out,
                    int32_t *w_out)
{
    if (n < 0 || m < 0 || F <= 0 || H <= 0 || mem_feature < 0 || mem_feature >= F) return -1;
    if (sm_on >= F || sm_off >= F || (sm_on >= 0) != (sm_off >= 0)) return -1;
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
#else
    (void)threads;
#endif
#pragma omp parallel for schedule(dynamic, 1)
    for (int i = 0; i < n; ++i) {
        const float *xu = x_on + (size_t)i * F;
        float *sig = (float *)malloc(sizeof(float) * (size_t)(m > 0 ? m : 1));
        if (wide) score_row_wide(xu, x_off, m, F, H, sm_on, sm_off, W1, b1, W2, b2, W3, b3, sig);
        else      score_row_narrow(xu, x_off, m, F, H, sm_on, sm_off, W1, b1, W2, b2, W3, b3, sig);
        for (int j = 0; j < m; ++j) {
            if (sigma_out) sigma_out[(size_t)i * m + j] = sig[j];
            if (w_out) {
                float q = rintf(sig[j] * scale);          /* float product, round half to even */
                if (q < 0.0f) q = 0.0f;
                if (q > scale) q = scale;
                int32_t w = (int32_t)q;
                float mem = xu[mem_feature] + x_off[(size_t)j * F + mem_feature];
                if (mem > mem_limit) w = ORC_INFEASIBLE;
                w_out[(size_t)i * m + j] = w;
            }
        }
        free(sig);
    }
    return 0;
}

int orc_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------------
 * Maximum-weight bipartite matching, exact (the role the paper gives the
 * Kuhn-Munkres algorithm: "find the optimal maximum weighted bipartite
 * matching", O(|V|^3)).
 *
 * A matching is a set of disjoint feasible edges; it need not cover every
 * row or column (the paper's worked example has 2 online and 3 offline
 * workloads).  All weights are >= 0, so the problem equals the row-perfect
 * assignment on w'[i][j] = W[i][j] if feasible else 0 (n <= m): any matching
 * extends to a row-perfect assignment by zero entries, and any row-perfect
 * assignment restricts to a matching of the same weight.  That assignment is
 * solved as a minimum-cost problem on c = -w' by successive shortest
 * augmenting paths with potentials, one new row per stage.
 *
 * Outputs: row2col[n] (-1 where the row stays unmatched or sits on an
 * infeasible entry), duals u[n], v[m] >= 0 with u_i + v_j >= w'_ij everywhere,
 * equality on assigned entries and v_j = 0 on unassigned columns, and
 * *total = sum of matched weights.
 * ---------------------------------------------------------------------- */
int orc_max_weight_matching(const int32_t *W, int n, int m, int64_t ldw,
                            int32_t *row2col, int64_t *u_out, int64_t *v_out, int64_t *total)
{
    if (n < 0 || m < 0 || n > m || ldw < m) return -1;
    const int64_t INF = INT64_MAX / 4;
    /* 1-based arrays; column 0 is the virtual start column of each stage */
    int64_t *u = (int64_t *)calloc((size_t)n + 1, sizeof(int64_t));
    int64_t *v = (int64_t *)calloc((size_t)m + 1, sizeof(int64_t));
    int64_t *minv = (int64_t *)malloc(sizeof(int64_t) * ((size_t)m + 1));
    int *p = (int *)calloc((size_t)m + 1, sizeof(int));     /* p[j] = row assigned to column j */
    int *way = (int *)calloc((size_t)m + 1, sizeof(int));
    char *used = (char *)malloc((size_t)m + 1);

    for (int i = 1; i <= n; ++i) {
        p[0] = i;
        int j0 = 0;
        for (int j = 0; j <= m; ++j) { minv[j] = INF; used[j] = 0; }
        do {
            used[j0] = 1;
            int i0 = p[j0], j1 = 0;
            int64_t delta = INF;
            const int32_t *row = W + (size_t)(i0 - 1) * ldw;
            for (int j = 1; j <= m; ++j) {
                if (used[j]) continue;
                int64_t wij = row[j - 1] == ORC_INFEASIBLE ? 0 : (int64_t)row[j - 1];
                int64_t cur = -wij - u[i0] - v[j];            /* reduced cost of (i0, j) */
                if (cur < minv[j]) { minv[j] = cur; way[j] = j0; }
                if (minv[j] < delta) { delta = minv[j]; j1 = j; }
            }
            for (int j = 0; j <= m; ++j) {
                if (used[j]) { u[p[j]] += delta; v[j] -= delta; }
                else minv[j] -= delta;
            }
            j0 = j1;
        } while (p[j0] != 0);
        do {                                                   /* flip the augmenting path */
            int j1 = way[j0];
            p[j0] = p[j1];
            j0 = j1;
        } while (j0);
    }

    /* Potentials of the minimisation satisfy u_i + v_j <= c_ij with v_j <= 0;
     * negate them for the maximisation and shift so that min_j V_j = 0. */
    int64_t shift = 0;
    if (m > 0) {
        shift = -v[1];
        for (int j = 2; j <= m; ++j) if (-v[j] < shift) shift = -v[j];
    }
    for (int j = 1; j <= m; ++j) v_out[j - 1] = -v[j] - shift;
    for (int i = 1; i <= n; ++i) u_out[i - 1] = -u[i] + shift;

    int64_t sum = 0;
    for (int i = 0; i < n; ++i) row2col[i] = -1;
    for (int j = 1; j <= m; ++j) {
        if (p[j] == 0) continue;
        int32_t w = W[(size_t)(p[j] - 1) * ldw + (j - 1)];
        if (w != ORC_INFEASIBLE) { row2col[p[j] - 1] = j - 1; sum += w; }
    }
    *total = sum;
    free(u); free(v); free(minv); free(p); free(way); free(used);
    return 0;
}

/* ------------------------------------------------------------------------
 * The same optimum by definition: enumerate every way of giving each row
 * either nothing or a feasible column no earlier row took.  n <= m <= 10.
 * ---------------------------------------------------------------------- */
static void enumerate(const int32_t *W, int n, int m, int64_t ldw, int i, unsigned taken,
                      int64_t sum, int32_t *cur, int64_t *best, int32_t *best_map)
{
    if (i == n) {
        if (sum > *best) { *best = sum; memcpy(best_map, cur, sizeof(int32_t) * (size_t)n); }
        return;
    }
    cur[i] = -1;
    enumerate(W, n, m, ldw, i + 1, taken, sum, cur, best, best_map);
    for (int j = 0; j < m; ++j) {
        int32_t w = W[(size_t)i * ldw + j];
        if ((taken >> j) & 1u || w == ORC_INFEASIBLE) continue;
        cur[i] = j;
        enumerate(W, n, m, ldw, i + 1, taken | (1u << j), sum + w, cur, best, best_map);
    }
    cur[i] = -1;
}

int orc_brute_force(const int32_t *W, int n, int m, int64_t ldw, int32_t *row2col, int64_t *total)
{
    if (n < 0 || m < 0 || n > 10 || m > 10 || ldw < m) return -1;
    int32_t cur[10], best_map[10];
    int64_t best = -1;
    for (int i = 0; i < n; ++i) { cur[i] = -1; best_map[i] = -1; }
    enumerate(W, n, m, ldw, 0, 0u, 0, cur, &best, best_map);
    for (int i = 0; i < n; ++i) row2col[i] = best_map[i];
    *total = best;
    return 0;
}

/* ------------------------------------------------------------------------
 * Optimality certificate by linear-programming duality.
 *
 * The matching LP (maximise the sum of chosen edge weights, every workload
 * in at most one chosen edge) has the dual: minimise sum u + sum v subject to
 * u_i + v_j >= w_ij on every feasible edge, u, v >= 0.  Any dual-feasible
 * (u, v) bounds every matching from above.  Duals may be given in units of
 * 1/K of a weight unit (K >= 1 integer): then u_i + v_j >= K * w_ij, and
 * since every matching weight is an integer, 0 <= D - K*P < K proves that
 * the matching of weight P is optimal.  K = 1 is the textbook statement
 * "reduced costs >= 0 and primal = dual".
 *
 * Returns 0 and fills *primal, *dual when everything holds; otherwise a
 * positive code naming the first failed condition:
 *   1 row2col out of range / not injective     2 matched pair infeasible
 *   3 negative dual                            4 a feasible edge with u_i+v_j < K*w_ij
 *   5 gap D - K*P outside [0, K)               -1 bad arguments
 * ---------------------------------------------------------------------- */
int orc_check_certificate(const int32_t *W, int n, int m, int64_t ldw, const int32_t *row2col,
                          const int64_t *u, const int64_t *v, int64_t K,
                          int64_t *primal, int64_t *dual)
{
    if (n < 0 || m < 0 || ldw < m || K < 1) return -1;
    char *taken = (char *)calloc((size_t)m + 1, 1);
    int64_t P = 0, D = 0;
    int bad = 0;
    for (int i = 0; i < n && !bad; ++i) {
        int j = row2col[i];
        if (j == -1) continue;
        if (j < 0 || j >= m || taken[j]) { bad = 1; break; }
        taken[j] = 1;
        int32_t w = W[(size_t)i * ldw + j];
        if (w == ORC_INFEASIBLE || w < 0) { bad = 2; break; }
        P += w;
    }
    free(taken);
    if (bad) return bad;
    for (int i = 0; i < n; ++i) { if (u[i] < 0) return 3; D += u[i]; }
    for (int j = 0; j < m; ++j) { if (v[j] < 0) return 3; D += v[j]; }
    int violated = 0;
#pragma omp parallel for reduction(| : violated)
    for (int i = 0; i < n; ++i) {
        const int32_t *row = W + (size_t)i * ldw;
        for (int j = 0; j < m; ++j) {
            if (row[j] == ORC_INFEASIBLE) continue;
            if (u[i] + v[j] < K * (int64_t)row[j]) violated |= 1;
        }
    }
    if (violated) return 4;
    *primal = P;
    *dual = D;
    if (D - K * P < 0 || D - K * P >= K) return 5;
    return 0;
}
