/*
 * oob_oracle.c -- plain CPU oracle of the pipeline-template planning dynamic
 * program (Section 4.1 of the Oobleck paper: node specification 4.1.1 and
 * GPU-stage mapping 4.1.2, Eq. 1-4, and the coverage theorem of Appendix A).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is slow on purpose, follows the paper's
 * steps in the paper's order and notation, and shares no code with the HIP
 * library.  Only tests, the smoke check and the benchmark's CPU-baseline leg
 * may load it; the product path never does.
 *
 * Arithmetic: int64 nanoseconds and bytes throughout.
 *
 * Notation.  L layers, M GPUs per node, N_b microbatches, cap bytes per GPU.
 * A state is (S', u, v, delta): layers [u, v) cut into S' stages on the device
 * set delta.  A device set is either G(g), 1 <= g <= M-1 ("g GPUs inside one
 * node"), or A(a), a >= 1 ("a whole nodes").  Index: delta = g-1 for G(g),
 * delta = M-2+a for A(a).
 *
 * Readings taken where the paper is silent or inconsistent (each is listed in
 * the design notes of the repository):
 *   - intervals are half open; the right sub-problem of a split at k is [k, v)
 *     (Eq. 1 and 3 print k+1, which would skip a layer);
 *   - k* is 0-indexed: only then does Eq. 2 at S'=1, N_b=4 give the 2(F+B) of
 *     Eq. 4;
 *   - ties for the slowest stage go to the smallest stage index;
 *   - ties between candidates go to the smallest (s, k, m) in that order, and
 *     between stage counts to the smallest S;
 *   - N_b is the caller's microbatch count at every level; N_b = 0 selects
 *     the paper's own planning-time choice N_b = 4 S' per state;
 *   - states with S' > N_b do not exist;
 *   - a multi-node device set is split at node granularity only, a single node
 *     is split into GPU counts (Section 4.1.2, time-complexity paragraph);
 *   - a stage fits iff ceil(sum of its layers' bytes / d) <= cap; a stage that
 *     is not the last one of the model pays boundary_ns of its last layer.
 *   parity unpinned by the paper: the memory rule and the boundary term are
 *   this build's definitions (the paper's Eq. 1-4 contain neither).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_FORBIDDEN ((int64_t)1 << 62) /* profile entry: this d not allowed */

typedef struct {
    int64_t T1, T3, tmax;
    int32_t kstar;
    int32_t s, k, m; /* winning split: stages, layer index, devices of the left half */
    int32_t exists;
} orec;

typedef struct oob_oracle {
    int L, M, n_max, Nb, D, Smax;
    int64_t cap;
    int64_t *PT;   /* [(M+1)][(L+1)] prefix sums of F+B for d GPUs            */
    int32_t *PF;   /* [(M+1)][(L+1)] prefix counts of forbidden entries       */
    int64_t *PM;   /* [L+1] prefix sums of bytes                              */
    int64_t *X;    /* [L] boundary ns                                         */
    orec **tab;    /* [(Smax+1) * D] -> (L+1)*(L+1) records, or NULL          */
    int64_t states, candidates, evaluated;
} oob_oracle;

/* ---- device sets ------------------------------------------------------- */
static int is_G(const oob_oracle *o, int delta) { return delta < o->M - 1; }
static int nodes_of(const oob_oracle *o, int delta) { return delta - (o->M - 2); }
static int delta_G(const oob_oracle *o, int g) { (void)o; return g - 1; }
static int delta_A(const oob_oracle *o, int a) { return o->M - 2 + a; }
/* GPUs of a device set that lies inside one node (G(g) or A(1)). */
static int gpus_single(const oob_oracle *o, int delta) {
    return is_G(o, delta) ? delta + 1 : o->M;
}

/* Which (S', delta) exist at all (Section 4.1.2, "Choosing the number of
 * stages": no stage spans nodes, so a whole-node set of a nodes needs at least
 * a stages; every GPU is used, so it has at most a*M; inside a node at most
 * one stage per GPU). */
static int valid_state(const oob_oracle *o, int S, int delta) {
    if (S < 1 || S > o->L) return 0;
    if (o->Nb > 0 && S > o->Nb) return 0;
    if (delta < 0 || delta >= o->D) return 0;
    if (is_G(o, delta)) return S <= delta + 1;
    int a = nodes_of(o, delta);
    return a <= S && S <= (int64_t)a * o->M;
}

static int64_t nb_of(const oob_oracle *o, int S) { return o->Nb > 0 ? o->Nb : 4 * (int64_t)S; }

static orec *block(const oob_oracle *o, int S, int delta) { return o->tab[(size_t)S * o->D + delta]; }
static orec *at(const oob_oracle *o, int S, int delta, int u, int v) {
    orec *b = block(o, S, delta);
    return b ? &b[(size_t)u * (o->L + 1) + v] : NULL;
}

/* Eq. 4: one stage of layers [u, v) on d GPUs of one node. */
static int stage_exists(const oob_oracle *o, int u, int v, int d, int64_t *t) {
    const int W = o->L + 1;
    if (o->PF[d * W + v] - o->PF[d * W + u] != 0) return 0; /* a layer forbids this d */
    int64_t bytes = o->PM[v] - o->PM[u];
    int64_t per_gpu = (bytes + d - 1) / d;
    if (per_gpu > o->cap) return 0;
    *t = o->PT[d * W + v] - o->PT[d * W + u] + (v < o->L ? o->X[v - 1] : 0);
    return 1;
}

/* Total iteration time of a record under its own stage count (T1 + T2 + T3,
 * with T2 of Eq. 2). */
static int64_t total_of(const oob_oracle *o, int S, const orec *r) {
    return r->T1 + (nb_of(o, S) - S + r->kstar - 1) * r->tmax + r->T3;
}

static void solve_state(oob_oracle *o, int S, int delta, int u, int v,
                        int64_t *cand, int64_t *eval) {
    orec *out = at(o, S, delta, u, v);
    out->exists = 0;
    if (S == 1) { /* conquer */
        int64_t t;
        if (stage_exists(o, u, v, gpus_single(o, delta), &t)) {
            out->T1 = out->T3 = out->tmax = t;
            out->kstar = 0; out->s = out->k = out->m = 0;
            out->exists = 1;
        }
        return;
    }
    /* divide: iterate s, then k, then m, ascending; keep the first strict minimum */
    const int multi = !is_G(o, delta) && nodes_of(o, delta) >= 2;
    const int units = multi ? nodes_of(o, delta) : gpus_single(o, delta);
    int64_t bestT = 0;
    const int64_t nb = nb_of(o, S);
    for (int s = 1; s <= S - 1; ++s) {
        for (int k = u + s; k <= v - (S - s); ++k) {
            for (int m = 1; m <= units - 1; ++m) {
                int dl = multi ? delta_A(o, m) : delta_G(o, m);
                int dr = multi ? delta_A(o, units - m) : delta_G(o, units - m);
                if (!valid_state(o, s, dl) || !valid_state(o, S - s, dr)) continue;
                ++*cand;
                const orec *A = at(o, s, dl, u, k);
                const orec *B = at(o, S - s, dr, k, v);
                if (!A->exists || !B->exists) continue; /* a missing child is skipped, never added */
                ++*eval;
                int64_t T1 = A->T1 + B->T1;                      /* Eq. 1 */
                int64_t tmax, T3; int32_t kstar;
                if (A->tmax >= B->tmax) {                        /* slowest stage in the left half */
                    tmax = A->tmax; kstar = A->kstar; T3 = A->T3 + B->T1;   /* Eq. 3, first case */
                } else {
                    tmax = B->tmax; kstar = s + B->kstar; T3 = B->T3;       /* Eq. 3, second case */
                }
                int64_t T2 = (nb - S + kstar - 1) * tmax;        /* Eq. 2 */
                int64_t T = T1 + T2 + T3;
                if (!out->exists || T < bestT) {
                    bestT = T;
                    out->T1 = T1; out->T3 = T3; out->tmax = tmax; out->kstar = kstar;
                    out->s = s; out->k = k; out->m = m; out->exists = 1;
                }
            }
        }
    }
}

/* ---- public C entry points (loaded through ctypes by the tests) --------- */

void oob_oracle_destroy(oob_oracle *o) {
    if (!o) return;
    if (o->tab) {
        for (size_t i = 0; i < (size_t)(o->Smax + 1) * o->D; ++i) free(o->tab[i]);
        free(o->tab);
    }
    free(o->PT); free(o->PF); free(o->PM); free(o->X);
    free(o);
}

/* Builds every table.  fwd/bwd: [L*M], entry l*M + (d-1).  threads <= 0 keeps
 * the OpenMP default.  Returns NULL on bad arguments or allocation failure. */
oob_oracle *oob_oracle_create(const int64_t *fwd, const int64_t *bwd, const int64_t *mem,
                              const int64_t *bnd, int L, int n_max, int M, int Nb,
                              int64_t cap, int threads) {
    if (L < 1 || n_max < 1 || M < 1 || Nb < 0 || cap <= 0) return NULL;
    oob_oracle *o = (oob_oracle *)calloc(1, sizeof(*o));
    if (!o) return NULL;
    o->L = L; o->M = M; o->n_max = n_max; o->Nb = Nb; o->cap = cap;
    o->D = M - 1 + n_max;
    int64_t smax = L;
    if ((int64_t)n_max * M < smax) smax = (int64_t)n_max * M;
    if (Nb > 0 && Nb < smax) smax = Nb;
    o->Smax = (int)smax;
    const int W = L + 1;
    o->PT = (int64_t *)calloc((size_t)(M + 1) * W, sizeof(int64_t));
    o->PF = (int32_t *)calloc((size_t)(M + 1) * W, sizeof(int32_t));
    o->PM = (int64_t *)calloc(W, sizeof(int64_t));
    o->X = (int64_t *)calloc(L, sizeof(int64_t));
    o->tab = (orec **)calloc((size_t)(o->Smax + 1) * o->D, sizeof(orec *));
    if (!o->PT || !o->PF || !o->PM || !o->X || !o->tab) { oob_oracle_destroy(o); return NULL; }
    for (int d = 1; d <= M; ++d)
        for (int l = 0; l < L; ++l) {
            int64_t F = fwd[(size_t)l * M + d - 1], B = bwd[(size_t)l * M + d - 1];
            int forb = (F >= ORACLE_FORBIDDEN || B >= ORACLE_FORBIDDEN);
            o->PT[d * W + l + 1] = o->PT[d * W + l] + (forb ? 0 : F + B);
            o->PF[d * W + l + 1] = o->PF[d * W + l] + forb;
        }
    for (int l = 0; l < L; ++l) { o->PM[l + 1] = o->PM[l] + mem[l]; o->X[l] = bnd[l]; }
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
#else
    (void)threads;
#endif
    for (int S = 1; S <= o->Smax; ++S) {
        for (int delta = 0; delta < o->D; ++delta) {
            if (!valid_state(o, S, delta)) continue;
            orec *b = (orec *)calloc((size_t)W * W, sizeof(orec));
            if (!b) { oob_oracle_destroy(o); return NULL; }
            o->tab[(size_t)S * o->D + delta] = b;
        }
        int64_t st = 0, cand = 0, eval = 0;
        /* states of one level only read lower levels, so they are independent */
#pragma omp parallel for collapse(2) schedule(dynamic, 1) reduction(+ : st, cand, eval)
        for (int delta = 0; delta < o->D; ++delta)
            for (int u = 0; u < L; ++u) {
                if (!valid_state(o, S, delta)) continue;
                for (int v = u + S; v <= L; ++v) {
                    ++st;
                    solve_state(o, S, delta, u, v, &cand, &eval);
                }
            }
        o->states += st; o->candidates += cand; o->evaluated += eval;
    }
    return o;
}

int oob_oracle_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

int oob_oracle_smax(const oob_oracle *o) { return o->Smax; }
int oob_oracle_ndelta(const oob_oracle *o) { return o->D; }
int64_t oob_oracle_states(const oob_oracle *o) { return o->states; }
int64_t oob_oracle_candidates(const oob_oracle *o) { return o->candidates; }
int64_t oob_oracle_evaluated(const oob_oracle *o) { return o->evaluated; }
int oob_oracle_valid(const oob_oracle *o, int S, int delta) { return valid_state(o, S, delta); }

/* Copies the records of one (S', delta) block into [(L+1)*(L+1)] arrays indexed
 * u*(L+1)+v.  T is the record's total under its own S'.  Returns 0 when the
 * pair (S', delta) is not valid. */
int oob_oracle_get_block(const oob_oracle *o, int S, int delta, int32_t *exists, int64_t *T,
                         int64_t *T1, int64_t *T3, int64_t *tmax, int32_t *kstar,
                         int32_t *s, int32_t *k, int32_t *m) {
    if (!valid_state(o, S, delta)) return 0;
    const orec *b = block(o, S, delta);
    size_t n = (size_t)(o->L + 1) * (o->L + 1);
    for (size_t i = 0; i < n; ++i) {
        exists[i] = b[i].exists;
        T[i] = b[i].exists ? total_of(o, S, &b[i]) : 0;
        T1[i] = b[i].T1; T3[i] = b[i].T3; tmax[i] = b[i].tmax; kstar[i] = b[i].kstar;
        s[i] = b[i].s; k[i] = b[i].k; m[i] = b[i].m;
    }
    return 1;
}

/* Writes the stages of state (S', u, v, delta) left to right. */
static void expand(const oob_oracle *o, int S, int u, int v, int delta,
                   int32_t *begin, int32_t *gpus, int *pos) {
    if (S == 1) {
        begin[*pos] = u; gpus[*pos] = gpus_single(o, delta); ++*pos;
        return;
    }
    const orec *r = at(o, S, delta, u, v);
    const int multi = !is_G(o, delta) && nodes_of(o, delta) >= 2;
    const int units = multi ? nodes_of(o, delta) : gpus_single(o, delta);
    int dl = multi ? delta_A(o, r->m) : delta_G(o, r->m);
    int dr = multi ? delta_A(o, units - r->m) : delta_G(o, units - r->m);
    expand(o, r->s, u, r->k, dl, begin, gpus, pos);
    expand(o, S - r->s, r->k, v, dr, begin, gpus, pos);
}

/* One template per node count n in [n_min, n_min+count) ("Choosing the number
 * of stages"): the stage count S in [n, min(L, nM, N_b)] whose state
 * (S, 0, L, A(n)) has the smallest total, smallest S on ties.
 * stage_gpus of template i starts at stage_off[i]; stage_begin (S+1 entries,
 * the last one is L) starts at stage_off[i] + i. */
void oob_oracle_templates(const oob_oracle *o, int n_min, int count, int32_t *feasible,
                          int32_t *S_out, int32_t *kstar, int64_t *T, int64_t *T1, int64_t *T2,
                          int64_t *T3, int64_t *tmax, int32_t *stage_off, int32_t *stage_begin,
                          int32_t *stage_gpus) {
    int off = 0;
    for (int i = 0; i < count; ++i) {
        int n = n_min + i;
        stage_off[i] = off;
        feasible[i] = 0; S_out[i] = 0; kstar[i] = 0;
        T[i] = T1[i] = T2[i] = T3[i] = tmax[i] = 0;
        const orec *best = NULL; int bestS = 0; int64_t bestT = 0;
        if (n <= o->n_max) {
            for (int S = n; S <= o->Smax; ++S) {
                int delta = delta_A(o, n);
                if (!valid_state(o, S, delta) || o->L < S) continue;
                const orec *r = at(o, S, delta, 0, o->L);
                if (!r->exists) continue;
                int64_t t = total_of(o, S, r);
                if (!best || t < bestT) { best = r; bestS = S; bestT = t; }
            }
        }
        if (!best) continue;
        feasible[i] = 1; S_out[i] = bestS; kstar[i] = best->kstar;
        T[i] = bestT; T1[i] = best->T1; T3[i] = best->T3; tmax[i] = best->tmax;
        T2[i] = (nb_of(o, bestS) - bestS + best->kstar - 1) * best->tmax;
        int pos = 0;
        expand(o, bestS, 0, o->L, delta_A(o, n), stage_begin + off + i, stage_gpus + off, &pos);
        stage_begin[off + i + bestS] = o->L;
        off += bestS;
    }
    stage_off[count] = off;
}

/* Node specification (Section 4.1.1) and the coverage guarantee (Appendix A).
 * n0 = smallest feasible node count; the template sizes are the consecutive
 * feasible counts n0..n_hi; N = n_hi + f*n0 (the largest template is N - f*n0).
 * hdr = {n0, n_hi, p, N, p > n0-1, lo, covered_theorem, covered_tail} where the
 * array maxpipes covers N' = lo..N, lo = min((f+1) n0, max(1, N-f)), and holds
 * the largest number of pipelines whose sizes sum to N' (0: no such sum).
 * covered_theorem: every N' in [(f+1) n0, N] has >= f+1 pipelines;
 * covered_tail: every N' in [max(1, N-f), N] is a sum of template sizes.
 * Coin-change recursion of Section 4.2.1 reduced to the largest count. */
void oob_oracle_coverage(const int32_t *feasible, int n_min, int count, int f,
                         int32_t *hdr, int32_t *maxpipes, int maxpipes_len) {
    for (int i = 0; i < 8; ++i) hdr[i] = 0;
    for (int i = 0; i < maxpipes_len; ++i) maxpipes[i] = 0;
    int i0 = -1;
    for (int i = 0; i < count; ++i) if (feasible[i]) { i0 = i; break; }
    if (i0 < 0) return;
    int i1 = i0;
    while (i1 + 1 < count && feasible[i1 + 1]) ++i1;
    int n0 = n_min + i0, n_hi = n_min + i1, p = n_hi - n0 + 1;
    int N = n_hi + f * n0;
    int lo_thm = (f + 1) * n0;
    int lo_tail = N - f < 1 ? 1 : N - f;
    int lo = lo_thm < lo_tail ? lo_thm : lo_tail;
    int *best = (int *)malloc(sizeof(int) * (size_t)(N + 1));
    best[0] = 0;
    for (int x = 1; x <= N; ++x) {
        best[x] = -1;
        for (int c = n0; c <= n_hi; ++c)
            if (x - c >= 0 && best[x - c] >= 0 && best[x - c] + 1 > best[x]) best[x] = best[x - c] + 1;
    }
    int thm = 1, tail = 1;
    for (int x = lo; x <= N; ++x) {
        int cnt = best[x] < 0 ? 0 : best[x];
        if (x - lo < maxpipes_len) maxpipes[x - lo] = cnt;
        if (x >= lo_thm && cnt < f + 1) thm = 0;
        if (x >= lo_tail && cnt < 1) tail = 0;
    }
    free(best);
    hdr[0] = n0; hdr[1] = n_hi; hdr[2] = p; hdr[3] = N; hdr[4] = p > n0 - 1;
    hdr[5] = lo; hdr[6] = thm; hdr[7] = tail;
}
