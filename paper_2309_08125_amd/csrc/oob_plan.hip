// MI355X (gfx950) pipeline-template planner: kernels and host driver behind the C ABI of
// include/oob_plan.h.  Method: Section 4.1 of the Oobleck paper (node specification 4.1.1,
// GPU-stage mapping 4.1.2 with Eq. 1-4, coverage theorem of Appendix A).
//
// Arithmetic.  Inputs and outputs are int64.  Inside the tables every time is held as an
// IEEE double: gfx950 issues 64-bit floating add / min / compare at full rate (one VALU
// instruction each) while a 64-bit integer add or compare takes two or more, and doubles are
// exact for integers below 2^53.  The set-up kernel proves the bound (every cost the
// recursion can form stays below 2^52 ns, about 52 days) or reports OOB_EOVERFLOW, so the
// results are bit-identical to int64 arithmetic.
//
// What a state stores.  With r = S' - s and children A = (s, u, k, left set),
// B = (r, k, v, right set), Eq. 1-3 give the candidate's total
//     slowest stage in A (A.tmax >= B.tmax):  T = A.T + cl * A.tmax + 2 * B.T1
//     slowest stage in B:                     T = A.T1 + B.T + cr * B.tmax
// where X.T is the child's own total under its own stage count, and (cl, cr) = (-r, 0) when
// N_b is the caller's microbatch count or (3r, 4s) when N_b = 4 S' per state.  So the hot
// loop needs only (T, T1, tmax) per child; T3 and k* are carried per state for the output.
#include <hip/hip_runtime.h>
#include <math.h>
#include <new>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "oob_layout.h"
#include "oob_plan.h"

namespace oob {

constexpr double kNone = __builtin_huge_val(); // total of a state that does not exist
constexpr long long kExactBound = 1LL << 52;

// Device view of the workspace.
struct Tables {
    Shape sh;
    long long *lvl_base; // [Smax+2] first element of level S'
    long long *PT;       // [(M+1)*(L+1)] prefix sums of F+B for d GPUs (row d)
    int *PF;             // [(M+1)*(L+1)] prefix counts of forbidden entries
    long long *PM;       // [L+1] prefix sums of bytes
    double *T, *T1, *tmax, *T3;
    int *kstar, *choice;
    int *stack;          // [count*(Smax+1)*4] backtracking stacks
};

__device__ __forceinline__ long long elem(const Tables &t, int S, int delta, int i, int j) {
    const int n = t.sh.L - S + 1;
    return t.lvl_base[S] + ((long long)(delta - dlo_of(S, t.sh.M)) * n + i) * n + j;
}

// ---------------------------------------------------------------------------------------
// Set-up: prefix sums (Eq. 4's sums become differences), input validation, level offsets.
// One block; thread d-1 scans the profile row of d GPUs.
// ---------------------------------------------------------------------------------------
__global__ void k_setup(Tables t, oob_profile prof, int *status) {
    const int L = t.sh.L, M = t.sh.M, W = L + 1;
    __shared__ long long s_worst[OOB_MAX_GPUS + 1];
    __shared__ int s_bad;
    if (threadIdx.x == 0) s_bad = 0;
    __syncthreads();
    const int d = threadIdx.x + 1;
    if (d <= M) {
        long long acc = 0, worst = 0;
        int forb = 0, bad = 0;
        t.PT[d * W] = 0;
        t.PF[d * W] = 0;
        for (int l = 0; l < L; ++l) {
            const long long F = prof.fwd_ns[(size_t)l * M + d - 1], B = prof.bwd_ns[(size_t)l * M + d - 1];
            if (F < 0 || B < 0) bad = 1;
            const int fb = (F >= OOB_FORBIDDEN || B >= OOB_FORBIDDEN);
            if (!fb) { acc += F + B; if (acc >= kExactBound) { bad = 2; acc = 0; } }
            forb += fb;
            t.PT[d * W + l + 1] = acc;
            t.PF[d * W + l + 1] = forb;
        }
        worst = acc;
        s_worst[d] = worst;
        if (bad) atomicMax(&s_bad, bad);
    }
    if (threadIdx.x == blockDim.x - 1) { // bytes, boundary terms, level offsets
        long long acc = 0, xs = 0;
        int bad = 0;
        t.PM[0] = 0;
        for (int l = 0; l < L; ++l) {
            const long long mb = prof.mem_bytes[l], x = prof.boundary_ns[l];
            if (mb < 0 || x < 0 || mb >= OOB_FORBIDDEN || acc + mb >= OOB_FORBIDDEN) bad = 1;
            if (x >= kExactBound || xs + x >= kExactBound) bad = imax(bad, 2); else xs += x;
            acc += mb;
            t.PM[l + 1] = acc;
        }
        s_worst[0] = xs;
        if (bad) atomicMax(&s_bad, bad);
        long long base = 0;
        for (int S = 1; S <= t.sh.Smax + 1; ++S) {
            t.lvl_base[S] = base;
            const int n = L - S + 1, nd = dhi_of(S, M, t.sh.n_max) - dlo_of(S, M) + 1;
            if (S <= t.sh.Smax && nd > 0) base += (long long)nd * n * n;
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int st = OOB_OK;
        if (s_bad == 1) st = OOB_EINVAL;
        else if (s_bad == 2) st = OOB_EOVERFLOW;
        else {
            // Every quantity the recursion forms is at most (N_b + 4 Smax + 4) * w, where w bounds
            // the sum of all stage times of any pipeline; the sum over d of the row totals plus all
            // boundary terms is such a w (loose, never too small).
            long long worst = s_worst[0];
            for (int dd = 1; dd <= M; ++dd) {
                worst += s_worst[dd];
                if (worst >= kExactBound) worst = kExactBound;
            }
            const long long nb = t.sh.Nb > 0 ? t.sh.Nb : 4LL * t.sh.Smax;
            const long long mult = nb + 4LL * t.sh.Smax + 4;
            if (worst >= kExactBound / mult) st = OOB_EOVERFLOW;
        }
        *status = st;
    }
}

// Stage time and feasibility of layers [u, v) on d GPUs of one node (Eq. 4; memory rule:
// ceil(bytes / d) <= cap; boundary term for a stage that is not the model's last).
__device__ __forceinline__ bool stage_time(const Tables &t, const long long *X, int u, int v, int d,
                                           long long *out) {
    const int W = t.sh.L + 1;
    if (t.PF[d * W + v] - t.PF[d * W + u] != 0) return false;
    const long long bytes = t.PM[v] - t.PM[u];
    if ((bytes + d - 1) / d > t.sh.cap) return false;
    *out = t.PT[d * W + v] - t.PT[d * W + u] + (v < t.sh.L ? X[v - 1] : 0);
    return true;
}

// ---------------------------------------------------------------------------------------
// Level 1 ("Conquer", Eq. 4): one thread per (delta, i, j) of the level-1 blocks.
// ---------------------------------------------------------------------------------------
__global__ void k_level1(Tables t, const long long *X) {
    const int L = t.sh.L, M = t.sh.M, n = L;
    const long long total = (long long)M * n * n;
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int j = (int)(idx % n), i = (int)((idx / n) % n), delta = (int)(idx / ((long long)n * n));
    const long long o = t.lvl_base[1] + idx;
    double T = kNone, T1 = kNone, tm = 0.0, T3 = 0.0;
    if (j >= i) {
        const int d = delta < M - 1 ? delta + 1 : M;
        long long st;
        if (stage_time(t, X, i, j + 1, d, &st)) {
            const double nb = t.sh.Nb > 0 ? (double)t.sh.Nb : 4.0;
            T1 = tm = T3 = (double)st;
            T = T1 + (nb - 2.0) * tm + T3; // Eq. 2 with S' = 1, k* = 0
        }
    }
    t.T[o] = T; t.T1[o] = T1; t.tmax[o] = tm; t.T3[o] = T3;
    t.kstar[o] = 0; t.choice[o] = 0;
}

// ---------------------------------------------------------------------------------------
// Levels S' >= 2 ("Divide", Eq. 1-3), plain version: one thread per state, candidates in
// the order s, k, m with a strict-minimum update (so the smallest (T, s, k, m) wins).
// ---------------------------------------------------------------------------------------
__global__ void k_combine_simple(Tables t, int Sp) {
    const int L = t.sh.L, M = t.sh.M, n = L - Sp + 1;
    const int dlo = dlo_of(Sp, M), nd = dhi_of(Sp, M, t.sh.n_max) - dlo + 1;
    const long long total = (long long)nd * n * n;
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int j = (int)(idx % n), i = (int)((idx / n) % n), delta = dlo + (int)(idx / ((long long)n * n));
    const long long o = t.lvl_base[Sp] + idx;
    double best = kNone;
    int bs = 0, bp = 0, bm = 0;
    if (j >= i) {
        const Family fam = family_of(delta, M);
        for (int s = 1; s < Sp; ++s) {
            const int r = Sp - s;
            int mlo, mhi;
            m_range(fam.fam_base, fam.units, s, r, M, &mlo, &mhi);
            if (mlo > mhi) continue;
            const double cl = t.sh.Nb > 0 ? -(double)r : 3.0 * r, cr = t.sh.Nb > 0 ? 0.0 : 4.0 * s;
            for (int p = i; p <= j; ++p) {          // k = p + s
                for (int m = mlo; m <= mhi; ++m) {
                    const long long oa = elem(t, s, fam.fam_base + m, i, p);
                    const long long ob = elem(t, r, fam.fam_base + fam.units - m, p + s, j + s);
                    const double aT = t.T[oa], aT1 = t.T1[oa], am = t.tmax[oa];
                    const double bT = t.T[ob], bT1 = t.T1[ob], bmx = t.tmax[ob];
                    const double left = aT + cl * am + 2.0 * bT1;
                    const double right = aT1 + (bT + cr * bmx);
                    const double T = am >= bmx ? left : right;
                    if (T < best) { best = T; bs = s; bp = p; bm = m; }
                }
            }
        }
    }
    double T1 = kNone, tm = 0.0, T3 = 0.0;
    int ks = 0, ch = 0;
    if (best < kNone) {
        const Family fam = family_of(delta, M);
        const long long oa = elem(t, bs, fam.fam_base + bm, i, bp);
        const long long ob = elem(t, Sp - bs, fam.fam_base + fam.units - bm, bp + bs, j + bs);
        T1 = t.T1[oa] + t.T1[ob];
        if (t.tmax[oa] >= t.tmax[ob]) { tm = t.tmax[oa]; ks = t.kstar[oa]; T3 = t.T3[oa] + t.T1[ob]; }
        else                          { tm = t.tmax[ob]; ks = bs + t.kstar[ob]; T3 = t.T3[ob]; }
        ch = bs | ((bp + bs) << 10) | (bm << 21);
    }
    t.T[o] = best; t.T1[o] = T1; t.tmax[o] = tm; t.T3[o] = T3;
    t.kstar[o] = ks; t.choice[o] = ch;
}

// ---------------------------------------------------------------------------------------
// Template extraction ("Choosing the number of stages"): thread i handles n = n_min + i.
// ---------------------------------------------------------------------------------------
__global__ void k_pick(Tables t, oob_templates out) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= t.sh.count) return;
    const int L = t.sh.L, M = t.sh.M, n = t.sh.n_min + i, delta = M - 2 + n;
    double best = kNone;
    int bestS = 0;
    if (n <= t.sh.n_max)
        for (int S = n; S <= t.sh.Smax; ++S) {
            if (delta < dlo_of(S, M) || delta > dhi_of(S, M, t.sh.n_max)) continue;
            const double T = t.T[elem(t, S, delta, 0, L - S)];
            if (T < best) { best = T; bestS = S; }
        }
    out.feasible[i] = bestS > 0;
    out.S[i] = bestS;
    long long T = 0, T1 = 0, T2 = 0, T3 = 0, tm = 0;
    int ks = 0;
    if (bestS > 0) {
        const long long o = elem(t, bestS, delta, 0, L - bestS);
        T = (long long)best; T1 = (long long)t.T1[o]; T3 = (long long)t.T3[o];
        tm = (long long)t.tmax[o]; ks = t.kstar[o];
        const long long nb = t.sh.Nb > 0 ? t.sh.Nb : 4LL * bestS;
        T2 = (nb - bestS + ks - 1) * tm; // Eq. 2
    }
    out.T[i] = T; out.T1[i] = T1; out.T2[i] = T2; out.T3[i] = T3; out.tmax[i] = tm; out.kstar[i] = ks;
}

// Expands the stored (s, k, m) tree of each template left to right into stages.
__global__ void k_backtrack(Tables t, oob_templates out) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i > t.sh.count) return;
    int off = 0;
    for (int q = 0; q < i && q < t.sh.count; ++q) off += out.S[q];
    if (i == t.sh.count) { out.stage_off[i] = off; return; }
    out.stage_off[i] = off;
    const int S = out.S[i];
    if (S == 0) return;
    const int L = t.sh.L, M = t.sh.M;
    int *stk = t.stack + (size_t)i * (t.sh.Smax + 1) * 4;
    int *begin = out.stage_begin + off + i, *gpus = out.stage_gpus + off;
    int sp = 0, pos = 0;
    stk[0] = S; stk[1] = M - 2 + t.sh.n_min + i; stk[2] = 0; stk[3] = L; sp = 1;
    while (sp > 0 && pos < S) {
        --sp;
        const int Sq = stk[sp * 4], delta = stk[sp * 4 + 1], u = stk[sp * 4 + 2], v = stk[sp * 4 + 3];
        if (Sq == 1) {
            begin[pos] = u;
            gpus[pos] = delta < M - 1 ? delta + 1 : M;
            ++pos;
            continue;
        }
        const int ch = t.choice[elem(t, Sq, delta, u, v - Sq)];
        const int s = ch & 1023, k = (ch >> 10) & 2047, m = (ch >> 21) & 1023;
        const Family fam = family_of(delta, M);
        if (sp + 2 > t.sh.Smax + 1) break; // cannot happen: pending stages never exceed S
        // right half first so that the left half is expanded first
        stk[sp * 4] = Sq - s; stk[sp * 4 + 1] = fam.fam_base + fam.units - m; stk[sp * 4 + 2] = k; stk[sp * 4 + 3] = v; ++sp;
        stk[sp * 4] = s; stk[sp * 4 + 1] = fam.fam_base + m; stk[sp * 4 + 2] = u; stk[sp * 4 + 3] = k; ++sp;
    }
    begin[S] = L;
}

// ---------------------------------------------------------------------------------------
// Node specification and coverage (Section 4.1.1, Appendix A): one thread; the sizes are a
// run of consecutive integers, so "largest pipeline count summing to x" is a coin-change
// recursion over at most N <= n_max (f + 1) entries held in the backtracking scratch.
// ---------------------------------------------------------------------------------------
__global__ void k_coverage(Tables t, oob_templates out, int len) {
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    for (int q = 0; q < 8; ++q) out.cover_hdr[q] = 0;
    for (int q = 0; q < len; ++q) out.cover_maxpipes[q] = 0;
    const int cnt = t.sh.count, f = t.sh.f;
    int i0 = -1;
    for (int q = 0; q < cnt; ++q) if (out.feasible[q]) { i0 = q; break; }
    if (i0 < 0) return;
    int i1 = i0;
    while (i1 + 1 < cnt && out.feasible[i1 + 1]) ++i1;
    const int n0 = t.sh.n_min + i0, n_hi = t.sh.n_min + i1, p = n_hi - n0 + 1;
    const int N = n_hi + f * n0;
    const int lo_thm = (f + 1) * n0, lo_tail = N - f < 1 ? 1 : N - f;
    const int lo = lo_thm < lo_tail ? lo_thm : lo_tail;
    // best[x mod (n_hi+1)]: a ring is enough because x only looks back n_hi entries
    int *best = t.stack; // free again: k_backtrack has finished
    const int ring = n_hi + 1;
    int thm = 1, tail = 1;
    best[0] = 0;
    for (int x = 1; x <= N; ++x) {
        int b = -1;
        for (int c = n0; c <= n_hi && c <= x; ++c) {
            const int prev = best[(x - c) % ring];
            if (prev >= 0 && prev + 1 > b) b = prev + 1;
        }
        best[x % ring] = b;
        const int c = b < 0 ? 0 : b;
        if (x >= lo) {
            if (x - lo < len) out.cover_maxpipes[x - lo] = c;
            if (x >= lo_thm && c < f + 1) thm = 0;
            if (x >= lo_tail && c < 1) tail = 0;
        }
    }
    out.cover_hdr[0] = n0; out.cover_hdr[1] = n_hi; out.cover_hdr[2] = p; out.cover_hdr[3] = N;
    out.cover_hdr[4] = p > n0 - 1; out.cover_hdr[5] = lo; out.cover_hdr[6] = thm; out.cover_hdr[7] = tail;
}

// ---------------------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------------------
inline size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

// Elements of all level blocks for a shape.
long long table_elems(int L, int M, int n_max, int Nb) {
    const int Smax = smax_of(L, n_max, M, Nb);
    long long e = 0;
    for (int S = 1; S <= Smax; ++S) {
        const int n = L - S + 1, nd = dhi_of(S, M, n_max) - dlo_of(S, M) + 1;
        if (nd > 0) e += (long long)nd * n * n;
    }
    return e;
}

struct Carve {
    size_t lvl_base, PT, PF, PM, T, T1, tmax, T3, kstar, choice, stack, total;
};
// Byte offsets of the workspace arrays; sized for the handle's maxima so that a call with a
// smaller shape uses a prefix of each array.
Carve carve(int L, int nodes, int M) {
    Carve c;
    const long long E = table_elems(L, M, nodes, 0);
    const int Smax = smax_of(L, nodes, M, 0);
    size_t o = 0;
    c.lvl_base = o; o = align_up(o + sizeof(long long) * (OOB_MAX_L + 3));
    c.PT = o;       o = align_up(o + sizeof(long long) * (size_t)(M + 1) * (L + 1));
    c.PF = o;       o = align_up(o + sizeof(int) * (size_t)(M + 1) * (L + 1));
    c.PM = o;       o = align_up(o + sizeof(long long) * (size_t)(L + 1));
    c.T = o;        o = align_up(o + sizeof(double) * (size_t)E);
    c.T1 = o;       o = align_up(o + sizeof(double) * (size_t)E);
    c.tmax = o;     o = align_up(o + sizeof(double) * (size_t)E);
    c.T3 = o;       o = align_up(o + sizeof(double) * (size_t)E);
    c.kstar = o;    o = align_up(o + sizeof(int) * (size_t)E);
    c.choice = o;   o = align_up(o + sizeof(int) * (size_t)E);
    c.stack = o;    o = align_up(o + sizeof(int) * (size_t)nodes * (Smax + 1) * 4 + sizeof(int) * (size_t)(nodes + 2));
    c.total = o;
    return c;
}

// Structural work counts: states = records with v - u >= S'; candidates = (s, k, m) with both
// children valid.  A block with n = L-S'+1 has n(n+1)/2 states and n(n+1)(n+2)/6 (u, k, v)
// triples per (s, m).
void work_counts(const Shape &sh, long long *states, long long *cands) {
    long long st = 0, ca = 0;
    for (int S = 1; S <= sh.Smax; ++S) {
        const long long n = sh.L - S + 1;
        const int dlo = dlo_of(S, sh.M), dhi = dhi_of(S, sh.M, sh.n_max);
        for (int delta = dlo; delta <= dhi; ++delta) {
            st += n * (n + 1) / 2;
            if (S == 1) continue;
            const Family fam = family_of(delta, sh.M);
            long long pairs = 0;
            for (int s = 1; s < S; ++s) {
                int lo, hi;
                m_range(fam.fam_base, fam.units, s, S - s, sh.M, &lo, &hi);
                if (hi >= lo) pairs += hi - lo + 1;
            }
            ca += pairs * (n * (n + 1) * (n + 2) / 6);
        }
    }
    *states = st; *cands = ca;
}

} // namespace oob

using namespace oob;

struct oob_plan {
    int max_L, max_nodes, max_M;
    char *ws;
    size_t ws_bytes;
    Carve cv;
    long long max_elems; // capacity of each table array, in records
    Shape last;       // shape of the last call (for oob_plan_block)
    bool have_last;
    hipEvent_t ev_begin, ev_end; // optional: recorded around the level launches
    bool timed;
};

#define OOB_HIP_CHECK(expr)                                                                   \
    do {                                                                                      \
        hipError_t e_ = (expr);                                                               \
        if (e_ != hipSuccess) {                                                               \
            fprintf(stderr, "oob_plan: %s failed: %s\n", #expr, hipGetErrorString(e_));       \
            return OOB_EHIP;                                                                  \
        }                                                                                     \
    } while (0)

extern "C" int oob_plan_max_stages(int L, int n_max, int gpus_per_node, int microbatches) {
    if (L < 1 || n_max < 1 || gpus_per_node < 1 || microbatches < 0) return OOB_EINVAL;
    return smax_of(L, n_max, gpus_per_node, microbatches);
}

static bool dims_ok(int L, int nodes, int M) {
    return L >= 1 && L <= OOB_MAX_L && nodes >= 1 && nodes <= OOB_MAX_NODES && M >= 1 && M <= OOB_MAX_GPUS;
}

extern "C" size_t oob_plan_workspace_size(int max_L, int max_nodes, int max_gpus_per_node) {
    if (!dims_ok(max_L, max_nodes, max_gpus_per_node)) return 0;
    return carve(max_L, max_nodes, max_gpus_per_node).total;
}

extern "C" int oob_plan_create(oob_plan **h, int max_L, int max_nodes, int max_gpus_per_node,
                               void *dev_workspace, size_t workspace_bytes) {
    if (!h) return OOB_EINVAL;
    *h = nullptr;
    if (!dims_ok(max_L, max_nodes, max_gpus_per_node) || !dev_workspace) return OOB_EINVAL;
    if (((uintptr_t)dev_workspace & 255) != 0) return OOB_EINVAL;
    const Carve cv = carve(max_L, max_nodes, max_gpus_per_node);
    if (workspace_bytes < cv.total) return OOB_ECAPACITY;
    oob_plan *p = new (std::nothrow) oob_plan();
    if (!p) return OOB_EINVAL;
    p->max_L = max_L; p->max_nodes = max_nodes; p->max_M = max_gpus_per_node;
    p->ws = (char *)dev_workspace; p->ws_bytes = workspace_bytes; p->cv = cv; p->have_last = false;
    p->ev_begin = nullptr; p->ev_end = nullptr; p->timed = false;
    p->max_elems = table_elems(max_L, max_gpus_per_node, max_nodes, 0);
    *h = p;
    return OOB_OK;
}

extern "C" int oob_plan_destroy(oob_plan *h) {
    if (!h) return OOB_EINVAL;
    if (h->ev_begin) { hipEventDestroy(h->ev_begin); hipEventDestroy(h->ev_end); }
    delete h;
    return OOB_OK;
}

static Tables make_tables(const oob_plan *h, const Shape &sh) {
    Tables t;
    t.sh = sh;
    t.lvl_base = (long long *)(h->ws + h->cv.lvl_base);
    t.PT = (long long *)(h->ws + h->cv.PT);
    t.PF = (int *)(h->ws + h->cv.PF);
    t.PM = (long long *)(h->ws + h->cv.PM);
    t.T = (double *)(h->ws + h->cv.T);
    t.T1 = (double *)(h->ws + h->cv.T1);
    t.tmax = (double *)(h->ws + h->cv.tmax);
    t.T3 = (double *)(h->ws + h->cv.T3);
    t.kstar = (int *)(h->ws + h->cv.kstar);
    t.choice = (int *)(h->ws + h->cv.choice);
    t.stack = (int *)(h->ws + h->cv.stack);
    return t;
}

static bool out_ok(const oob_templates *o) {
    return o && o->feasible && o->S && o->kstar && o->T && o->T1 && o->T2 && o->T3 && o->tmax &&
           o->stage_off && o->stage_begin && o->stage_gpus && o->cover_hdr && o->cover_maxpipes &&
           o->status;
}

extern "C" int oob_plan_templates(oob_plan *h, const oob_profile *profile, int L, int n_min, int n_max,
                                  int gpus_per_node, int microbatches, int64_t mem_cap, int f,
                                  oob_templates *out, void *stream) {
    if (!h || !profile || !out_ok(out)) return OOB_EINVAL;
    if (!profile->fwd_ns || !profile->bwd_ns || !profile->mem_bytes || !profile->boundary_ns) return OOB_EINVAL;
    if (L < 1 || n_min < 1 || n_min > n_max || gpus_per_node < 1 || microbatches < 0 || f < 0 || mem_cap <= 0)
        return OOB_EINVAL;
    if (L > h->max_L || n_max > h->max_nodes || gpus_per_node > h->max_M) return OOB_ECAPACITY;
    if ((long long)n_max * ((long long)f + 1) > (1 << 24)) return OOB_ECAPACITY;
    Shape sh;
    sh.L = L; sh.M = gpus_per_node; sh.n_min = n_min; sh.n_max = n_max; sh.Nb = microbatches; sh.f = f;
    sh.cap = mem_cap; sh.count = n_max - n_min + 1;
    sh.Smax = smax_of(L, n_max, gpus_per_node, microbatches);
    if (table_elems(L, gpus_per_node, n_max, microbatches) > h->max_elems) return OOB_ECAPACITY;
    const Tables t = make_tables(h, sh);
    hipStream_t st = (hipStream_t)stream;
    work_counts(sh, (long long *)&out->states, (long long *)&out->candidates);

    hipLaunchKernelGGL(k_setup, dim3(1), dim3(OOB_MAX_GPUS + 1), 0, st, t, *profile, out->status);
    {
        const long long total = (long long)sh.M * L * L;
        hipLaunchKernelGGL(k_level1, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, t,
                           (const long long *)profile->boundary_ns);
    }
    if (h->ev_begin) OOB_HIP_CHECK(hipEventRecord(h->ev_begin, st));
    for (int S = 2; S <= sh.Smax; ++S) {
        const long long n = L - S + 1;
        const int nd = dhi_of(S, sh.M, sh.n_max) - dlo_of(S, sh.M) + 1;
        if (nd <= 0) continue;
        const long long total = nd * n * n;
        hipLaunchKernelGGL(k_combine_simple, dim3((unsigned)((total + 63) / 64)), dim3(64), 0, st, t, S);
    }
    if (h->ev_end) { OOB_HIP_CHECK(hipEventRecord(h->ev_end, st)); h->timed = true; }
    hipLaunchKernelGGL(k_pick, dim3((sh.count + 63) / 64), dim3(64), 0, st, t, *out);
    hipLaunchKernelGGL(k_backtrack, dim3((sh.count + 1 + 63) / 64), dim3(64), 0, st, t, *out);
    const int len = sh.count > f + 1 ? sh.count : f + 1;
    hipLaunchKernelGGL(k_coverage, dim3(1), dim3(64), 0, st, t, *out, len);
    OOB_HIP_CHECK(hipGetLastError());
    h->last = sh;
    h->have_last = true;
    return OOB_OK;
}

extern "C" int oob_plan_templates_batch(oob_plan *h, int count, const oob_profile *profiles, const int *L,
                                        const int *n_min, const int *n_max, const int *gpus_per_node,
                                        const int *microbatches, const int64_t *mem_cap, const int *f,
                                        oob_templates *outs, void *stream) {
    if (!h || count < 0 || (count > 0 && (!profiles || !L || !n_min || !n_max || !gpus_per_node ||
                                           !microbatches || !mem_cap || !f || !outs)))
        return OOB_EINVAL;
    for (int i = 0; i < count; ++i) {
        const int rc = oob_plan_templates(h, &profiles[i], L[i], n_min[i], n_max[i], gpus_per_node[i],
                                          microbatches[i], mem_cap[i], f[i], &outs[i], stream);
        if (rc != OOB_OK) return rc;
    }
    return OOB_OK;
}

extern "C" int oob_plan_level_timing(oob_plan *h, int enable) {
    if (!h) return OOB_EINVAL;
    if (enable && !h->ev_begin) {
        OOB_HIP_CHECK(hipEventCreate(&h->ev_begin));
        OOB_HIP_CHECK(hipEventCreate(&h->ev_end));
    } else if (!enable && h->ev_begin) {
        hipEventDestroy(h->ev_begin); hipEventDestroy(h->ev_end);
        h->ev_begin = h->ev_end = nullptr;
    }
    h->timed = false;
    return OOB_OK;
}

extern "C" int oob_plan_last_level_ms(oob_plan *h, float *ms) {
    if (!h || !ms || !h->ev_begin || !h->timed) return OOB_EINVAL;
    OOB_HIP_CHECK(hipEventSynchronize(h->ev_end));
    OOB_HIP_CHECK(hipEventElapsedTime(ms, h->ev_begin, h->ev_end));
    return OOB_OK;
}

extern "C" int oob_plan_block(const oob_plan *h, int S, int delta, oob_block_desc *desc) {
    if (!h || !desc || !h->have_last) return OOB_EINVAL;
    const Shape &sh = h->last;
    if (S < 1 || S > sh.Smax) return OOB_EINVAL;
    const int dlo = dlo_of(S, sh.M), dhi = dhi_of(S, sh.M, sh.n_max);
    if (delta < dlo || delta > dhi) return OOB_EINVAL;
    long long base = 0;
    for (int q = 1; q < S; ++q) {
        const long long n = sh.L - q + 1;
        const int nd = dhi_of(q, sh.M, sh.n_max) - dlo_of(q, sh.M) + 1;
        if (nd > 0) base += nd * n * n;
    }
    const long long n = sh.L - S + 1;
    desc->n = (int32_t)n;
    desc->elem_off = base + (long long)(delta - dlo) * n * n;
    desc->T_bytes = (int64_t)h->cv.T; desc->T1_bytes = (int64_t)h->cv.T1;
    desc->tmax_bytes = (int64_t)h->cv.tmax; desc->T3_bytes = (int64_t)h->cv.T3;
    desc->kstar_bytes = (int64_t)h->cv.kstar; desc->choice_bytes = (int64_t)h->cv.choice;
    return OOB_OK;
}
