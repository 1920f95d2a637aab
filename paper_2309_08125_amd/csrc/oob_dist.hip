// Batch distribution (Section 4.2.2, Eq. 6 of the Oobleck paper) and the choice of the plan by
// throughput, for gfx950.  One lane solves one plan, exactly.
//
// Method.  For a fixed level mu,  min sum_i (N_i T_i - mu)^2  over sum N_i = Q, N_i >= 1  is a
// separable convex allocation: rounding mu / T_i and then adding or removing microbatches one at
// a time where that is cheapest gives its optimum, and as mu grows the optimum changes by single
// exchanges of one microbatch from a faster to a slower pipeline, each at a level that is a ratio
// of integers.  Every allocation on that path is feasible for Eq. 6, and at mu = the mean of an
// optimum of Eq. 6 the path holds such an optimum (the sum of squares around the mean IS the
// variance, and no allocation has a smaller one), so the smallest variance met on the path is
// the minimum.  Any feasible allocation bounds the part of the path that matters: with V its
// sum of squared deviations, no pipeline of an optimum is further than sqrt(V) from the
// optimum's mean, hence that mean is within sqrt(V) of Q / sum_i (1 / T_i).
//
// Pipelines of one template have the same T and stay within one microbatch of each other, so the
// state of a plan is one total per template in use (at most 16), kept in LDS with one column
// per lane (192 bytes a lane; the templates' times are one table per workgroup); a template's
// donor is one of its fullest pipelines, its receiver one of its emptiest.  Products reach
// 2^124: all exact arithmetic is in 128-bit integers.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "oob_dist.h"
#include "oob_plan.h"

namespace oob_dist {

typedef __int128 i128;
constexpr int kLanes = 256; // plans per workgroup
constexpr int kT = OOB_DIST_MAX_TEMPLATES_IN_PLAN;
constexpr long long kMaxExchanges = 1ll << 24; // never reached (at most Q exchanges per template): every lane's loop ends

struct Args {
    const unsigned short *x;
    long long count, capacity;
    int p;
    const long long *tT;
    int Q;
    unsigned long long *vx;
    long long *slowest;
    unsigned short *base, *extra;
    int *status;
};

// One plan's state: column `lane` of arrays [kT][kLanes].  Template k of the plan has x pipelines;
// e of them hold n + 1 microbatches, the others n (0 <= e < x): no division in the loops.
struct Plan {
    const long long *tT;           // the workgroup's copy of the templates' times per microbatch
    unsigned short *j, *x, *n, *e; // template index; pipelines; see above
    int t, xs;                     // templates in use; pipelines in all
    __device__ long long Tk(int k) const { return tT[j[k * kLanes]]; }
    __device__ int xk(int k) const { return x[k * kLanes]; }
    __device__ int fullest(int k) const { return n[k * kLanes] + (e[k * kLanes] > 0); } // microbatches of a fullest pipeline
    __device__ int emptiest(int k) const { return n[k * kLanes]; }
    __device__ void take(int k) const { // one microbatch less for a fullest pipeline
        if (e[k * kLanes] > 0) e[k * kLanes] -= 1;
        else { n[k * kLanes] -= 1; e[k * kLanes] = (unsigned short)(xk(k) - 1); }
    }
    __device__ void give(int k) const { // one more for an emptiest pipeline
        if (e[k * kLanes] + 1 == xk(k)) { n[k * kLanes] += 1; e[k * kLanes] = 0; }
        else e[k * kLanes] += 1;
    }
};

// The optimum of the fixed-level problem at the integer level mu >= 0.
__device__ void allocate_at(const Plan &pl, long long mu, int Q) {
    long long tot = 0;
    for (int k = 0; k < pl.t; ++k) {
        const long long T = pl.Tk(k);
        long long n = (2 * mu + T) / (2 * T); // nearest integer to mu / T
        if (n < 1) n = 1;
        if (n > Q) n = Q;
        pl.n[k * kLanes] = (unsigned short)n;
        pl.e[k * kLanes] = 0;
        tot += n * pl.xk(k);
    }
    while (tot > Q) { // remove where it costs least: f(n-1) - f(n) = T^2 (1 - 2n) + 2 T mu, n = a fullest pipeline's
        int arg = -1;
        i128 best = 0;
        for (int k = 0; k < pl.t; ++k) {
            const int n = pl.fullest(k);
            if (n < 2) continue;
            const long long T = pl.Tk(k);
            const i128 c = (i128)T * T * (1 - 2 * n) + (i128)(2 * T) * mu;
            if (arg < 0 || c < best) { best = c; arg = k; }
        }
        if (arg < 0) break; // cannot happen: tot > Q >= pipelines, so some pipeline holds two
        pl.take(arg);
        --tot;
    }
    while (tot < Q) { // add where it costs least: f(n+1) - f(n) = T^2 (2n + 1) - 2 T mu, n = an emptiest pipeline's
        int arg = 0;
        i128 best = 0;
        for (int k = 0; k < pl.t; ++k) {
            const long long T = pl.Tk(k);
            const i128 c = (i128)T * T * (2 * pl.emptiest(k) + 1) - (i128)(2 * T) * mu;
            if (k == 0 || c < best) { best = c; arg = k; }
        }
        pl.give(arg);
        ++tot;
    }
}

// S1 = sum a_i, S2 = sum a_i^2 over the pipelines (a_i = N_i T_i).
__device__ void sums(const Plan &pl, i128 *S1, i128 *S2) {
    i128 s1 = 0, s2 = 0;
    for (int k = 0; k < pl.t; ++k) {
        const i128 T = pl.Tk(k);
        const int n = pl.n[k * kLanes], e = pl.e[k * kLanes]; // e pipelines hold n + 1, the others n
        const i128 lo = T * n, hi = T * (n + 1);
        s1 += lo * (pl.xk(k) - e) + hi * e;
        s2 += lo * lo * (pl.xk(k) - e) + hi * hi * e;
    }
    *S1 = s1; *S2 = s2;
}

__global__ void __launch_bounds__(kLanes) k_dist_solve(Args a) {
    HIP_DYNAMIC_SHARED(long long, s_tT) // [p]
    __shared__ unsigned short s_x[kT * kLanes], s_j[kT * kLanes], s_n[kT * kLanes], s_e[kT * kLanes];
    __shared__ unsigned short s_bn[kT * kLanes], s_be[kT * kLanes]; // the best allocation met so far
    const int lane = threadIdx.x;
    for (int j = lane; j < a.p; j += kLanes) s_tT[j] = a.tT[j];
    __syncthreads();
    const long long i = (long long)blockIdx.x * kLanes + lane;
    if (i >= a.count) return;
    Plan pl;
    pl.tT = s_tT; pl.j = s_j + lane; pl.x = s_x + lane; pl.n = s_n + lane; pl.e = s_e + lane;
    unsigned short *bn = s_bn + lane, *be = s_be + lane, *tj = s_j + lane;

    // the templates in use
    int t = 0, xs = 0, st = OOB_DIST_OK;
    for (int j = 0; j < a.p; ++j) {
        const int c = a.x[(long long)j * a.capacity + i];
        if (a.base) { a.base[(long long)j * a.capacity + i] = 0; a.extra[(long long)j * a.capacity + i] = 0; }
        if (!c || st != OOB_DIST_OK) continue;
        const long long T = a.tT[j];
        if (t == kT) { st = OOB_DIST_TOO_MANY_TEMPLATES; continue; }
        if (T < 1 || T > OOB_DIST_MAX_T) { st = OOB_DIST_BAD_TIME; continue; }
        pl.x[t * kLanes] = (unsigned short)c; tj[t * kLanes] = (unsigned short)j;
        xs += c;
        ++t;
    }
    if (st == OOB_DIST_OK && t == 0) st = OOB_DIST_NO_PIPELINE;
    if (st == OOB_DIST_OK && xs > a.Q) st = OOB_DIST_TOO_FEW_MICROBATCHES;
    a.status[i] = st;
    if (st != OOB_DIST_OK) {
        a.vx[2 * i] = 0; a.vx[2 * i + 1] = 0; a.slowest[i] = 0;
        return;
    }
    pl.t = t; pl.xs = xs;

    // the stretch of levels that can hold the optimum's mean
    double H = 0;
    for (int k = 0; k < t; ++k) H += (double)pl.xk(k) / (double)pl.Tk(k);
    const double L0 = (double)a.Q / H;
    allocate_at(pl, (long long)(L0 + 0.5), a.Q);
    i128 S1, S2;
    sums(pl, &S1, &S2);
    const double V = (double)((i128)xs * S2 - S1 * S1) / (double)xs; // sum of squared deviations of a feasible allocation
    const double R = sqrt(V) * (1.0 + 1e-9) + L0 * 1e-9 + 2.0;       // widened for the rounding of these few operations
    const long long mu_lo = L0 - R > 0 ? (long long)(L0 - R) : 0;
    const i128 mu_hi = (i128)(long long)(L0 + R) + 1;

    allocate_at(pl, mu_lo, a.Q);
    sums(pl, &S1, &S2);
    i128 best = (i128)xs * S2 - S1 * S1;
    for (int k = 0; k < t; ++k) { bn[k * kLanes] = pl.n[k * kLanes]; be[k * kLanes] = pl.e[k * kLanes]; }
    for (long long step = 0; step < kMaxExchanges; ++step) {
        // the next exchange: a microbatch of a fullest pipeline of template d (n_d of them) goes to an emptiest
        // pipeline of a slower template r (n_r): it pays from the level c / w on,
        // c = T_d^2 + T_r^2 - 2 T_d^2 n_d + 2 T_r^2 n_r,  w = 2 (T_r - T_d) > 0
        int bd = -1, br = -1;
        i128 bc = 0;
        long long bw = 1; // w < 2^37: a 64-bit factor keeps the two products of a comparison cheap
        for (int d = 0; d < t; ++d) {
            const int nd = pl.fullest(d);
            if (nd < 2) continue;
            const long long Td = pl.Tk(d);
            const i128 cd = (i128)Td * Td * (1 - 2 * nd);
            for (int r = 0; r < t; ++r) {
                const long long Tr = pl.Tk(r);
                if (Tr <= Td) continue;
                const i128 c = cd + (i128)Tr * Tr * (1 + 2 * pl.emptiest(r));
                const long long w = 2 * (Tr - Td);
                if (bd < 0 || c * bw < bc * w) { bc = c; bw = w; bd = d; br = r; }
            }
        }
        if (bd < 0 || bc > bw * mu_hi) break; // past the stretch
        const long long Td = pl.Tk(bd), Tr = pl.Tk(br);
        const int nd = pl.fullest(bd), nr = pl.emptiest(br);
        S1 += Tr - Td;
        S2 += (i128)Tr * Tr * (2 * nr + 1) - (i128)Td * Td * (2 * nd - 1);
        pl.take(bd);
        pl.give(br);
        const i128 v = (i128)xs * S2 - S1 * S1;
        if (v < best) {
            best = v;
            for (int k = 0; k < t; ++k) { bn[k * kLanes] = pl.n[k * kLanes]; be[k * kLanes] = pl.e[k * kLanes]; }
        }
    }

    long long slow = 0;
    for (int k = 0; k < t; ++k) {
        const int n = bn[k * kLanes], e = be[k * kLanes];
        const long long time = (long long)(n + (e > 0)) * pl.Tk(k);
        slow = time > slow ? time : slow;
        if (a.base) {
            a.base[(long long)tj[k * kLanes] * a.capacity + i] = (unsigned short)n;
            a.extra[(long long)tj[k * kLanes] * a.capacity + i] = (unsigned short)e;
        }
    }
    a.vx[2 * i] = (unsigned long long)best;
    a.vx[2 * i + 1] = (unsigned long long)(best >> 64);
    a.slowest[i] = slow;
}

// Plan choice: the smallest `slowest` among the solved plans of a group, the first of equals.
// A workgroup reduces one chunk of kChooseChunk consecutive plans of one group (lanes keep the
// first minimum of their strided share, waves and then the workgroup combine (value, index) pairs
// lexicographically) and merges its winner into best[group] with a compare-and-swap on the index:
// `slowest` does not change during the launch, so "is plan i better than the plan best[group]
// names now" is decided by reading both values, and the loop ends as soon as the entry names a plan
// that is at least as good.  k_dist_choose_init sets every entry to -1 ("no plan") first.
constexpr int kChooseThreads = 256, kChooseChunk = 2048;
__global__ void k_dist_choose_init(long long *best, int segments) {
    const int g = blockIdx.x * blockDim.x + threadIdx.x;
    if (g < segments) best[g] = -1;
}
__device__ __forceinline__ bool better(long long v, long long i, long long bv, long long bi) {
    return i >= 0 && (bi < 0 || v < bv || (v == bv && i < bi));
}
__global__ void __launch_bounds__(kChooseThreads) k_dist_choose(const long long *offsets, int segments,
                                                          const long long *slowest, const int *status,
                                                          long long *best) {
    __shared__ long long s_v[kChooseThreads / 64], s_i[kChooseThreads / 64];
    // this workgroup's chunk of the plans, cut to the plans the groups cover
    long long lo = offsets[0] + (long long)blockIdx.x * kChooseChunk;
    const long long all = offsets[segments], hi = lo + kChooseChunk < all ? lo + kChooseChunk : all;
    if (lo >= hi) return; // the same for the whole workgroup
    int g = 0;            // last group that starts at or before lo (empty groups before it are skipped)
    for (int a = 0, b = segments - 1; a <= b;) {
        const int mid = (a + b) >> 1;
        if (offsets[mid] <= lo) { g = mid; a = mid + 1; } else b = mid - 1;
    }
    for (; g < segments && lo < hi; ++g) { // every group that has plans in the chunk (uniform loop)
        const long long gend = offsets[g + 1], end = gend < hi ? gend : hi;
        if (end <= lo) continue;
        long long bv = 0, bi = -1;
        for (long long i = lo + threadIdx.x; i < end; i += kChooseThreads) // ascending: a lane keeps its first minimum
            if (status[i] == OOB_DIST_OK && (bi < 0 || slowest[i] < bv)) { bv = slowest[i]; bi = i; }
        for (int d = 32; d >= 1; d >>= 1) {
            const long long ov = __shfl_down(bv, d, 64), oi = __shfl_down(bi, d, 64);
            if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
        }
        __syncthreads(); // the previous group's partial results have been read
        if ((threadIdx.x & 63) == 0) { s_v[threadIdx.x >> 6] = bv; s_i[threadIdx.x >> 6] = bi; }
        __syncthreads();
        if (threadIdx.x == 0) {
            for (int w = 1; w < kChooseThreads / 64; ++w)
                if (better(s_v[w], s_i[w], bv, bi)) { bv = s_v[w]; bi = s_i[w]; }
            if (bi >= 0) {
                unsigned long long *slot = (unsigned long long *)&best[g];
                long long cur = (long long)atomicAdd(slot, 0ull); // coherent read of the entry
                while (better(bv, bi, cur >= 0 ? slowest[cur] : 0, cur)) {
                    const long long seen = (long long)atomicCAS(slot, (unsigned long long)cur, (unsigned long long)bi);
                    if (seen == cur) break;
                    cur = seen;
                }
            }
        }
        lo = end;
    }
}

} // namespace oob_dist

extern "C" int oob_dist_solve(const uint16_t *x, int64_t count, int64_t capacity, int p, const int64_t *template_T,
                              int Q, uint64_t *vx, int64_t *slowest, uint16_t *base, uint16_t *extra,
                              int32_t *status, void *stream) {
    using namespace oob_dist;
    if (!x || !template_T || !vx || !slowest || !status || (base == nullptr) != (extra == nullptr)) return OOB_EINVAL;
    if (count < 0 || capacity < count || p < 1 || p > OOB_DIST_MAX_TEMPLATES || Q < 1 || Q > OOB_DIST_MAX_Q) return OOB_EINVAL;
    if (count == 0) return OOB_OK;
    const long long blocks = (count + kLanes - 1) / kLanes;
    if (blocks > 0x7fffffffll) return OOB_EINVAL;
    Args a;
    a.x = x; a.count = count; a.capacity = capacity; a.p = p; a.tT = (const long long *)template_T; a.Q = Q;
    a.vx = (unsigned long long *)vx; a.slowest = (long long *)slowest; a.base = base; a.extra = extra; a.status = status;
    hipLaunchKernelGGL(k_dist_solve, dim3((unsigned)blocks), dim3(kLanes), (size_t)p * sizeof(long long), (hipStream_t)stream, a);
    return hipGetLastError() == hipSuccess ? OOB_OK : OOB_EHIP;
}

extern "C" int oob_dist_choose(const int64_t *offsets, int segments, int64_t count, const int64_t *slowest,
                               const int32_t *status, int64_t *best, void *stream) {
    using namespace oob_dist;
    if (!offsets || !slowest || !status || !best || segments < 0 || count < 0) return OOB_EINVAL;
    if (segments == 0) return OOB_OK;
    const long long chunks = (count + kChooseChunk - 1) / kChooseChunk;
    if (chunks > 0x7fffffffll) return OOB_EINVAL;
    hipLaunchKernelGGL(k_dist_choose_init, dim3((unsigned)((segments + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                       (long long *)best, segments);
    if (chunks > 0)
        hipLaunchKernelGGL(k_dist_choose, dim3((unsigned)chunks), dim3(kChooseThreads), 0, (hipStream_t)stream,
                           (const long long *)offsets, segments, (const long long *)slowest, status, (long long *)best);
    return hipGetLastError() == hipSuccess ? OOB_OK : OOB_EHIP;
}
