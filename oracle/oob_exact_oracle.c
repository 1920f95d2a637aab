/*
 * oob_exact_oracle.c -- TEST INFRASTRUCTURE ONLY (nothing in the product path may call it).
 *
 * The exact minimum of the pipeline cost of Section 4.1.2 over ALL explicit pipelines of a
 * template, which the paper's divide-and-conquer recursion (Eq. 1-3) only approximates.
 *
 * A pipeline for n nodes of M GPUs: stages 0..S-1 over contiguous layers, stage i on d_i <= M
 * GPUs, the stages filling node after node exactly.  With t_i the stage times, k* the first
 * slowest stage and tau = t_{k*}, the closed form of Eq. 1-4,
 *     C = sum_i t_i + (N_b - S + k* - 1) tau + sum_{i >= k*} t_i,
 * is the same as
 *     C = sum_{i < k*} t_i  +  N_b tau  +  sum_{i > k*} (2 t_i - tau),
 * so for a FIXED tau the stages before and after the slowest one contribute separately:
 *     Pre[p][D] = least sum of t over stage sequences that cover layers [0, p) on exactly the
 *                 first D GPUs, every t < tau   (strictly: k* is the FIRST slowest stage)
 *     Suf[p][E] = least sum of (2 t - tau) over sequences that cover [p, L) on exactly the last
 *                 E GPUs, every t <= tau
 * (a stage never crosses a node boundary; node boundaries are the multiples of M counted from
 * either end, the total being n M), and the minimum is taken over every stage (u, v, d) whose
 * time is tau and every place D it can start at:  Pre[u][D] + N_b tau + Suf[v][n M - D - d].
 * Stage time, memory rule and boundary term as in oob_oracle.c.
 *
 * Two functions.  oob_oracle_exact_minimum keeps no stage count in its tables: it is exact when the
 * limit S <= N_b cannot bind (N_b >= min(L, n M) for the template, or N_b = 4 S chosen per
 * pipeline, the paper's planning-time choice, Nb = 0 here) and otherwise the minimum over the larger
 * set of pipelines without the limit, a lower bound.  With N_b = 4 S the cost
 *     sum t + (4 S - S + k* - 1) tau + sum_{i >= k*} t_i  =  sum_{i < k*} (t_i + 4 tau) + 4 tau + sum_{i > k*} (2 t_i + 3 tau)
 * (3 S + k* + 1 = 4 k* + 4 + 3 (S - 1 - k*)) separates in the same way with other weights.
 * oob_oracle_exact_minimum_staged carries the stage count j as a third index of both tables
 * (plain sums of t), so that the limit k* + 1 + (stages after) <= N_b is part of the minimum:
 *     C = Pre[u][D][j1] + (N_b - j2) tau + 2 Suf[v][E][j2],            j1 + 1 + j2 <= N_b      (Nb > 0)
 *     C = Pre[u][D][j1] + (4 j1 + 4 + 3 j2) tau + 2 Suf[v][E][j2]                               (Nb = 0)
 * Plain loops, one tau after the other (OpenMP over tau for the timing of large cases).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define EXACT_FORBIDDEN ((int64_t)1 << 62)
#define EXACT_INF ((int64_t)1 << 61)

static int cmp_i64(const void *a, const void *b) {
    const int64_t x = *(const int64_t *)a, y = *(const int64_t *)b;
    return x < y ? -1 : x > y;
}

/* best[n - n_min] = the exact minimum for n nodes, or -1 if no pipeline exists.
 * Without the stage-count limit (see the header): exact for a template n when Nb = 0 or
 * Nb >= min(L, n M), a lower bound otherwise (which can be negative, once stages outnumber
 * microbatches, and then cannot be told from "no pipeline": use the number only where it is exact).
 * Returns the number of distinct tau tried, or -1 for arguments it does not take. */
int64_t oob_oracle_exact_minimum(const int64_t *fwd, const int64_t *bwd, const int64_t *mem, const int64_t *bnd,
                                 int L, int M, int n_min, int n_max, int Nb, int64_t cap, int64_t *best) {
    if (L < 1 || M < 1 || n_min < 1 || n_max < n_min || Nb < 0) return -1;
    /* weights of a stage before / after the slowest one and of the slowest one itself, in units of
     * (t, tau): Nb > 0: t, 2 t - tau, Nb tau;  Nb = 0 (N_b = 4 S): t + 4 tau, 2 t + 3 tau, 4 tau */
    const int64_t pre_tau = Nb > 0 ? 0 : 4, suf_tau = Nb > 0 ? -1 : 3, mid_tau = Nb > 0 ? Nb : 4;
    const int Dmax = n_max * M, count = n_max - n_min + 1;
    /* t[(u * (L + 1) + v) * M + d - 1] = time of stage [u, v) on d GPUs, -1 if impossible */
    int64_t *t = (int64_t *)malloc(sizeof(int64_t) * (size_t)(L + 1) * (L + 1) * M);
    int64_t *taus = (int64_t *)malloc(sizeof(int64_t) * (size_t)(L + 1) * (L + 1) * M);
    int64_t ntau = 0;
    for (int u = 0; u < L; ++u)
        for (int d = 1; d <= M; ++d) {
            int64_t time = 0, bytes = 0;
            int ok = 1;
            for (int v = u + 1; v <= L; ++v) {
                const int64_t f = fwd[(size_t)(v - 1) * M + d - 1], b = bwd[(size_t)(v - 1) * M + d - 1];
                if (f >= EXACT_FORBIDDEN || b >= EXACT_FORBIDDEN) ok = 0;
                time += ok ? f + b : 0;
                bytes += mem[v - 1];
                int64_t val = -1;
                if (ok && (bytes + d - 1) / d <= cap) val = time + (v < L ? bnd[v - 1] : 0);
                t[((size_t)u * (L + 1) + v) * M + d - 1] = val;
                if (val >= 0) taus[ntau++] = val;
            }
        }
    qsort(taus, (size_t)ntau, sizeof(int64_t), cmp_i64);
    int64_t nuniq = 0;
    for (int64_t i = 0; i < ntau; ++i)
        if (i == 0 || taus[i] != taus[i - 1]) taus[nuniq++] = taus[i];
    for (int i = 0; i < count; ++i) best[i] = EXACT_INF;

#pragma omp parallel
    {
        int64_t *Pre = (int64_t *)malloc(sizeof(int64_t) * (size_t)(L + 1) * (Dmax + 1));
        int64_t *Suf = (int64_t *)malloc(sizeof(int64_t) * (size_t)(L + 1) * (Dmax + 1));
        int64_t *mine = (int64_t *)malloc(sizeof(int64_t) * (size_t)count);
        for (int i = 0; i < count; ++i) mine[i] = EXACT_INF;
#pragma omp for schedule(dynamic, 1)
        for (int64_t it = 0; it < nuniq; ++it) {
            const int64_t tau = taus[it];
            for (size_t i = 0; i < (size_t)(L + 1) * (Dmax + 1); ++i) Pre[i] = Suf[i] = EXACT_INF;
            Pre[0] = 0;
            for (int p = 1; p <= L; ++p)
                for (int q = 0; q < p; ++q)
                    for (int d = 1; d <= M; ++d) {
                        const int64_t tt = t[((size_t)q * (L + 1) + p) * M + d - 1];
                        if (tt < 0 || tt >= tau) continue;
                        for (int D = 0; D + d <= Dmax; ++D) {
                            if (D % M + d > M) continue; /* would cross a node boundary */
                            const int64_t c = Pre[(size_t)q * (Dmax + 1) + D] + tt + pre_tau * tau;
                            if (c < Pre[(size_t)p * (Dmax + 1) + D + d]) Pre[(size_t)p * (Dmax + 1) + D + d] = c;
                        }
                    }
            Suf[(size_t)L * (Dmax + 1)] = 0;
            for (int p = L - 1; p >= 0; --p)
                for (int v = p + 1; v <= L; ++v)
                    for (int d = 1; d <= M; ++d) {
                        const int64_t tt = t[((size_t)p * (L + 1) + v) * M + d - 1];
                        if (tt < 0 || tt > tau) continue;
                        for (int E = d; E <= Dmax; ++E) {
                            if ((E - d) % M + d > M) continue;
                            const int64_t c = Suf[(size_t)v * (Dmax + 1) + E - d] + 2 * tt + suf_tau * tau;
                            if (c < Suf[(size_t)p * (Dmax + 1) + E]) Suf[(size_t)p * (Dmax + 1) + E] = c;
                        }
                    }
            for (int u = 0; u < L; ++u)
                for (int v = u + 1; v <= L; ++v)
                    for (int d = 1; d <= M; ++d) {
                        if (t[((size_t)u * (L + 1) + v) * M + d - 1] != tau) continue;
                        for (int n = n_min; n <= n_max; ++n)
                            for (int D = 0; D + d <= n * M; ++D) {
                                if (D % M + d > M) continue;
                                const int64_t a = Pre[(size_t)u * (Dmax + 1) + D], b = Suf[(size_t)v * (Dmax + 1) + n * M - D - d];
                                if (a >= EXACT_INF / 2 || b >= EXACT_INF / 2) continue;
                                const int64_t c = a + mid_tau * tau + b;
                                if (c < mine[n - n_min]) mine[n - n_min] = c;
                            }
                    }
        }
#pragma omp critical
        for (int i = 0; i < count; ++i)
            if (mine[i] < best[i]) best[i] = mine[i];
        free(Pre); free(Suf); free(mine);
    }
    for (int i = 0; i < count; ++i)
        if (best[i] >= EXACT_INF / 2) best[i] = -1;
    free(t); free(taus);
    return nuniq;
}

/* The same minimum with the stage count in the tables: exact for every Nb >= 1 (limit S <= Nb) and
 * for Nb = 0 (N_b = 4 S per pipeline).  best[n - n_min] = minimum for n nodes, -1 if no pipeline.
 * Tables of (L + 1) (Dmax + 1) (Smax + 1) entries per thread: small and middle sizes only. */
int64_t oob_oracle_exact_minimum_staged(const int64_t *fwd, const int64_t *bwd, const int64_t *mem, const int64_t *bnd,
                                        int L, int M, int n_min, int n_max, int Nb, int64_t cap, int64_t *best) {
    if (L < 1 || M < 1 || n_min < 1 || n_max < n_min || Nb < 0) return -1;
    const int Dmax = n_max * M, count = n_max - n_min + 1;
    int Smax = L < Dmax ? L : Dmax;
    if (Nb > 0 && Nb < Smax) Smax = Nb;
    const size_t W = (size_t)Dmax + 1, J = (size_t)Smax + 1;
    int64_t *t = (int64_t *)malloc(sizeof(int64_t) * (size_t)(L + 1) * (L + 1) * M);
    int64_t *taus = (int64_t *)malloc(sizeof(int64_t) * (size_t)(L + 1) * (L + 1) * M);
    int64_t ntau = 0;
    for (int u = 0; u < L; ++u)
        for (int d = 1; d <= M; ++d) {
            int64_t time = 0, bytes = 0;
            int ok = 1;
            for (int v = u + 1; v <= L; ++v) {
                const int64_t f = fwd[(size_t)(v - 1) * M + d - 1], b = bwd[(size_t)(v - 1) * M + d - 1];
                if (f >= EXACT_FORBIDDEN || b >= EXACT_FORBIDDEN) ok = 0;
                time += ok ? f + b : 0;
                bytes += mem[v - 1];
                int64_t val = -1;
                if (ok && (bytes + d - 1) / d <= cap) val = time + (v < L ? bnd[v - 1] : 0);
                t[((size_t)u * (L + 1) + v) * M + d - 1] = val;
                if (val >= 0) taus[ntau++] = val;
            }
        }
    qsort(taus, (size_t)ntau, sizeof(int64_t), cmp_i64);
    int64_t nuniq = 0;
    for (int64_t i = 0; i < ntau; ++i)
        if (i == 0 || taus[i] != taus[i - 1]) taus[nuniq++] = taus[i];
    for (int i = 0; i < count; ++i) best[i] = EXACT_INF;

#pragma omp parallel
    {
        /* Pre[(p W + D) J + j], Suf likewise: plain sums of stage times over j stages */
        int64_t *Pre = (int64_t *)malloc(sizeof(int64_t) * (size_t)(L + 1) * W * J);
        int64_t *Suf = (int64_t *)malloc(sizeof(int64_t) * (size_t)(L + 1) * W * J);
        int64_t *mine = (int64_t *)malloc(sizeof(int64_t) * (size_t)count);
        for (int i = 0; i < count; ++i) mine[i] = EXACT_INF;
#pragma omp for schedule(dynamic, 1)
        for (int64_t it = 0; it < nuniq; ++it) {
            const int64_t tau = taus[it];
            for (size_t i = 0; i < (size_t)(L + 1) * W * J; ++i) Pre[i] = Suf[i] = EXACT_INF;
            Pre[0] = 0; /* no layers, no GPUs, no stages */
            for (int p = 1; p <= L; ++p)
                for (int q = 0; q < p; ++q)
                    for (int d = 1; d <= M; ++d) {
                        const int64_t tt = t[((size_t)q * (L + 1) + p) * M + d - 1];
                        if (tt < 0 || tt >= tau) continue;
                        for (int D = 0; D + d <= Dmax; ++D) {
                            if (D % M + d > M) continue;
                            for (int j = 0; j < Smax; ++j) {
                                const int64_t c = Pre[((size_t)q * W + D) * J + j] + tt;
                                int64_t *dst = &Pre[((size_t)p * W + D + d) * J + j + 1];
                                if (c < *dst) *dst = c;
                            }
                        }
                    }
            Suf[((size_t)L * W) * J] = 0;
            for (int p = L - 1; p >= 0; --p)
                for (int v = p + 1; v <= L; ++v)
                    for (int d = 1; d <= M; ++d) {
                        const int64_t tt = t[((size_t)p * (L + 1) + v) * M + d - 1];
                        if (tt < 0 || tt > tau) continue;
                        for (int E = d; E <= Dmax; ++E) {
                            if ((E - d) % M + d > M) continue;
                            for (int j = 0; j < Smax; ++j) {
                                const int64_t c = Suf[((size_t)v * W + E - d) * J + j] + tt;
                                int64_t *dst = &Suf[((size_t)p * W + E) * J + j + 1];
                                if (c < *dst) *dst = c;
                            }
                        }
                    }
            for (int u = 0; u < L; ++u)
                for (int v = u + 1; v <= L; ++v)
                    for (int d = 1; d <= M; ++d) {
                        if (t[((size_t)u * (L + 1) + v) * M + d - 1] != tau) continue;
                        for (int n = n_min; n <= n_max; ++n)
                            for (int D = 0; D + d <= n * M; ++D) {
                                if (D % M + d > M) continue;
                                for (int j1 = 0; j1 < Smax; ++j1) {
                                    const int64_t a = Pre[((size_t)u * W + D) * J + j1];
                                    if (a >= EXACT_INF / 2) continue;
                                    for (int j2 = 0; j1 + 1 + j2 <= Smax; ++j2) {
                                        const int64_t b = Suf[((size_t)v * W + n * M - D - d) * J + j2];
                                        if (b >= EXACT_INF / 2) continue;
                                        const int64_t coef = Nb > 0 ? (int64_t)Nb - j2 : 4 * (int64_t)j1 + 4 + 3 * (int64_t)j2;
                                        const int64_t c = a + coef * tau + 2 * b;
                                        if (c < mine[n - n_min]) mine[n - n_min] = c;
                                    }
                                }
                            }
                    }
        }
#pragma omp critical
        for (int i = 0; i < count; ++i)
            if (mine[i] < best[i]) best[i] = mine[i];
        free(Pre); free(Suf); free(mine);
    }
    for (int i = 0; i < count; ++i)
        if (best[i] >= EXACT_INF / 2) best[i] = -1;
    free(t); free(taus);
    return nuniq;
}
