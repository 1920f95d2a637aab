// Exact minimum of the pipeline cost (Section 4.1.2 of the Oobleck paper; the closed form of
// Eq. 1-4) over all explicit pipelines, for gfx950.
//
// With k* the first slowest stage and tau its time,
//     C = sum_{i<k*} t_i + N_b tau + sum_{i>k*} (2 t_i - tau)                        (N_b given)
//     C = sum_{i<k*} (t_i + 4 tau) + 4 tau + sum_{i>k*} (2 t_i + 3 tau)              (N_b = 4 S)
// so around a FIXED slowest stage (u, v, d) the stages before and after it are two independent
// shortest-path problems.  A stage never crosses a node boundary and the stages fill node after
// node, so a pipeline around (u, v, d) is: `a` whole nodes covering layers [0, q), then g GPUs of the
// slowest stage's node covering [q, u), the stage itself, the remaining h = M - g - d GPUs of that
// node covering [v, x), and b whole nodes covering [x, L); n = a + 1 + b.
//
// k_exact_lds (the fast path; everything in LDS, times as exact integers in doubles).  One
// workgroup per slowest stage.  Phase 1, per wave and start layer q, no workgroup barrier: the
// one-node table G_q[p][g] = least cost of covering [q, p) with stages on exactly the first g GPUs
// of a node; it yields W[q][p] = G_q[p][M] (a whole node) and GU[q][g] = G_q[u][g].  Phase 2: the
// node-level recurrence NP_a[p] = min_q NP_{a-1}[q] + W[q][p] and PreU[a][g] = min_q NP_a[q] +
// GU[q][g], one barrier per node count.  The same two phases mirrored for the layers after v,
// then every (template, a, g) combination.  Global memory is read for the stage times only (one
// table for the whole call, resident in L2).
//
// k_exact_flat (tables in the caller's workspace, int64): the plain recurrence over (layer, GPUs
// used [, stages used]).  It serves shapes whose tables exceed LDS and, with the stage count as a
// third index (plain sums of t; the coefficient of tau follows from the counts at the end), the
// limit S <= N_b: oob_exact_minimum_staged.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

#include "oob_exact.h"

namespace oob_exact {

constexpr int kThreads = 256;       // k_exact_flat
constexpr int kFlatSlots = 2048;    // its workgroups in flight at most, each with tables of its own
constexpr long long kInf = 1ll << 61;
constexpr long long kForbidden = 1ll << 62;
constexpr long long kDoubleExact = 1ll << 52;
constexpr double kNone = __builtin_huge_val();
constexpr size_t kLdsLimit = 160 * 1024;

struct Args {
    oob_profile prof;
    int L, M, n_min, n_max, Nb, Dmax, Smax;
    long long cap;
    long long limit;      // every cost must stay below this (2^52 for the LDS path, 2^61 otherwise)
    long long *t;         // [(u (L+1) + v) M + d-1] stage times, -1: impossible
    double *tds, *tdp;    // the same as doubles, laid out for the two walks of the fast path: tds[(u M + d-1)(L+1) + v]
                          // (a stage out of u: v runs along a row), tdp[(v M + d-1)(L+1) + u] (a stage into v: u runs along a row)
    long long *slots;     // k_exact_flat: [slots][2][(L+1)][(Dmax+1)][J]
    unsigned long long *best; // per template: smallest cost so far
    unsigned *counter;    // work counter of k_exact_lds
    int *status;
};

inline size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }
__host__ __device__ inline size_t table_entries(int L, int M) { return (size_t)(L + 1) * (L + 1) * M; }
// the tables of doubles carry one more row, every entry "impossible", and a few entries of padding: the
// walks of the fast path read up to three entries past their end, and idle lanes walk the extra row
__host__ __device__ inline size_t dtable_entries(int L, int M) { return table_entries(L, M) + (size_t)(L + 1) + 8; }
inline size_t head_bytes(int L, int M) { return 256 + align_up(8 * table_entries(L, M)) + 2 * align_up(8 * dtable_entries(L, M)); }
constexpr int kGPad = 3; // rows of "impossible" in front of a one-node table

// LDS of k_exact_lds for `nw` waves, in bytes (all arrays 8-byte entries; see the kernel).
__host__ __device__ inline size_t tri(int L) { return (size_t)L * (L + 1) / 2; }
inline size_t lds_bytes(int L, int M, int n_max, int count, int nw) {
    const size_t n = tri(L) + (size_t)(L + 1) * M + 4 * (size_t)(L + 1) + 2 * (size_t)n_max * M +
                     ((size_t)(L + 1) * M + 1) / 2 + (size_t)(L + 1) / 2 + 1 + L + count +
                     (size_t)nw * (L + 1 + kGPad) * (M + 1);
    return 8 * n + 64;
}
inline int lds_waves(int L, int M, int n_max, int count) { // 0: does not fit
    for (int nw : {16, 12, 8, 4, 2}) // the one-node phase is bound by the latency of a table row: as many waves as fit
        if (lds_bytes(L, M, n_max, count, nw) <= kLdsLimit) return nw;
    return 0;
}

// Clears the result and validates the magnitudes: every cost is at most mult * w, w = the sum over
// the layers of the slowest allowed F + B of the layer plus its boundary term (a bound on the sum
// of all stage times of any pipeline), mult = N_b + 2 (4 S_max + 2 when N_b = 4 S).  status =
// OOB_EOVERFLOW unless that stays below the limit of the path.  One workgroup; runs before
// k_exact_stages, which only ever sets the status to OOB_EINVAL.
__global__ void __launch_bounds__(kThreads) k_exact_init(Args a) {
    __shared__ long long s_sum[kThreads];
    const int count = a.n_max - a.n_min + 1;
    for (int i = threadIdx.x; i < count; i += kThreads) a.best[i] = 0x7FF0000000000000ull; // +inf as a double, huge as an integer
    if (threadIdx.x == 0) *a.counter = 0;
    const long long *fwd = (const long long *)a.prof.fwd_ns, *bwd = (const long long *)a.prof.bwd_ns;
    const long long *bnd = (const long long *)a.prof.boundary_ns;
    long long acc = 0;
    for (int l = threadIdx.x; l < a.L; l += kThreads) {
        long long worst = 0;
        for (int d = 1; d <= a.M; ++d) {
            const long long f = fwd[(size_t)l * a.M + d - 1], b = bwd[(size_t)l * a.M + d - 1];
            if (f < 0 || b < 0 || f >= kForbidden || b >= kForbidden) continue;
            const long long fb = (f >= kInf || b >= kInf) ? kInf : f + b;
            worst = fb > worst ? fb : worst;
        }
        const long long x = bnd[l];
        if (x > 0) worst = (x >= kInf || worst >= kInf) ? kInf : worst + x;
        acc = (acc + worst >= kInf || worst >= kInf) ? kInf : acc + worst;
    }
    s_sum[threadIdx.x] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        long long w = 0;
        for (int i = 0; i < kThreads; ++i) w = (w + s_sum[i] >= kInf) ? kInf : w + s_sum[i];
        const long long mult = (a.Nb > 0 ? (long long)a.Nb : 4ll * a.Smax) + 2;
        *a.status = w >= a.limit / mult ? OOB_EOVERFLOW : OOB_OK;
    }
}

// Every entry of the two tables of doubles, the extra row and the padding included: "impossible".
__global__ void k_exact_fill(Args a) {
    const size_t n = dtable_entries(a.L, a.M);
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
        a.tds[i] = kNone;
        a.tdp[i] = kNone;
    }
}

// Stage times of all (u, v, d): one thread per (u, d) walks v.  A negative profile entry sets the
// status to OOB_EINVAL (every writer stores the same value, so the order does not matter).
__global__ void k_exact_stages(Args a) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= a.L * a.M) return;
    const int u = i / a.M, d = i % a.M + 1;
    const long long *fwd = (const long long *)a.prof.fwd_ns, *bwd = (const long long *)a.prof.bwd_ns;
    const long long *mem = (const long long *)a.prof.mem_bytes, *bnd = (const long long *)a.prof.boundary_ns;
    long long time = 0, bytes = 0;
    bool ok = true, bad = false;
    for (int v = u + 1; v <= a.L; ++v) {
        const long long f = fwd[(size_t)(v - 1) * a.M + d - 1], b = bwd[(size_t)(v - 1) * a.M + d - 1];
        if (f < 0 || b < 0 || mem[v - 1] < 0 || bnd[v - 1] < 0) bad = true;
        if (f >= kForbidden || b >= kForbidden) ok = false;
        time += ok ? f + b : 0;
        bytes += mem[v - 1];
        long long val = -1;
        if (ok && (bytes + d - 1) / d <= a.cap) val = time + (v < a.L ? bnd[v - 1] : 0);
        const size_t o = ((size_t)u * (a.L + 1) + v) * a.M + d - 1;
        a.t[o] = val;
        if (val >= 0) { // an impossible stage keeps the fill value of the tables of doubles
            a.tds[((size_t)u * a.M + d - 1) * (a.L + 1) + v] = (double)val;
            a.tdp[((size_t)v * a.M + d - 1) * (a.L + 1) + u] = (double)val;
        }
    }
    if (bad) atomicExch(a.status, OOB_EINVAL);
}

// ---------------------------------------------------------------------------------------------
// The fast path.
// ---------------------------------------------------------------------------------------------
// What one wave has written to LDS is read by its other lanes: program order of the LDS operations
// of a wave is execution order, the fences keep the compiler from moving them.
__device__ __forceinline__ void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}
// Minimum over aligned groups of 4 / 8 consecutive lanes, in every lane of the group, with data-parallel
// moves (quad permutations 1,0,3,2 and 2,3,0,1; then the mirror image within each half row, which
// hands every lane a lane of the other quad of its group of eight).
template <int CTRL> __device__ __forceinline__ double dpp_f64(double x) {
    int lo = __double2loint(x), hi = __double2hiint(x);
    lo = __builtin_amdgcn_update_dpp(lo, lo, CTRL, 0xF, 0xF, false);
    hi = __builtin_amdgcn_update_dpp(hi, hi, CTRL, 0xF, 0xF, false);
    return __hiloint2double(hi, lo);
}
__device__ __forceinline__ double min4(double x) {
    x = fmin(x, dpp_f64<0xB1>(x));
    return fmin(x, dpp_f64<0x4E>(x));
}
__device__ __forceinline__ double min8(double x) {
    x = min4(x);
    return fmin(x, dpp_f64<0x141>(x));
}

struct Lds {
    double *W;    // [tri(L)]  one whole node covering [q, p), q < p: index q L - q (q-1)/2 + p - q - 1
    double *GU;   // [(L+1)][M]  g GPUs (entry g, 1 <= g < M) of a node covering [q, u) / (mirrored) [v, x)
    double *NP;   // [2][2][L+1]  per side: node-level tables of the previous and the current node count
    double *PU;   // [n_max][M]  PreU[a][g]
    double *SV;   // [n_max][M]  SufV[b][h]
    int *lo;      // [(L+1)][M]  first (prefix) / last (suffix) layer a stage into / out of p can reach
    int *lomin;   // [L+1]       the extreme of lo over the GPU counts
    double *bnd;  // [L]
    unsigned long long *best; // [count]
    double *G;    // [waves][(L+1)][(M+1)]
};
__device__ __forceinline__ size_t widx(int q, int p, int L) { return (size_t)q * L - (size_t)q * (q - 1) / 2 + (p - q - 1); }

// The two sides of the slowest stage [u, v).  MIRROR = false: the layers [0, e) before it (e = u); a
// one-node table starts at layer q and grows to the right, a stage [q', p) into p costs t + ptau * tau
// and needs t < tau.  MIRROR = true: the layers [e, L) after it (e = v); a one-node table ends at
// layer q and grows to the left, a stage [p, w) out of p costs 2 t + stau * tau and needs t <= tau.
// Result per side: OUT[c][g] = least cost of covering the side with c whole nodes and g more GPUs
// next to the slowest stage, g = 0 .. M-1.  The two sides use disjoint parts of every table that is
// indexed by layers (W, GU, lo, lomin), so they run side by side.

// Reach of a stage into / out of layer p on dd GPUs (entry i = p M + dd - 1), by bisection.
template <bool MIRROR>
__device__ __forceinline__ int side_reach(const Args &a, const Lds &s, int p, int dd, double tau) {
    const int L = a.L, M = a.M;
    if (!MIRROR) {
        // [x, p) only gets slower and heavier as x goes down (impossible at the far end): the stages
        // with t < tau are x = r .. p-1
        int lo = 0, hi = p; // answer in [lo, hi]; hi = p: none
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            const double tt = a.tdp[((size_t)p * M + dd - 1) * (L + 1) + mid];
            if (tt < tau) hi = mid; else lo = mid + 1;
        }
        return lo;
    }
    // [p, w) as w goes up: impossible stays impossible and the time without the boundary term only
    // grows: those stages are w = p+1 .. r
    int lo = p, hi = L; // answer in [lo, hi]; lo = p: none
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        const double tt = a.tds[((size_t)p * M + dd - 1) * (L + 1) + mid];
        if (tt - (mid < L ? s.bnd[mid - 1] : 0.0) <= tau) lo = mid; else hi = mid - 1;
    }
    return lo;
}

// One-node table of start layer q (one wave): rows, then its contribution to W and GU.
template <bool MIRROR>
__device__ void one_node_table(const Args &a, const Lds &s, int e, int q, double tau, double wt, double add, double *G) {
    const int L = a.L, M = a.M, lane = threadIdx.x & 63, gi = lane >> 3, di = lane & 7;
    // row r of G = layer q + r (prefix) / q - r (suffix); row 0: nothing covered
    for (int g = lane; g <= M; g += 64) G[g] = g == 0 ? 0.0 : kNone;
    wave_sync();
    const int rows = MIRROR ? q - e : e - q;
    int lastfin = q; // the layer farthest from q that some number of GPUs can be made to reach
    for (int r = 1; r <= rows; ++r) {
        const int p = MIRROR ? q - r : q + r;
        // farthest layer any stage of this row reaches (the same in every lane: say so, the loops below
        // then count in scalar registers)
        const int far = __builtin_amdgcn_readfirstlane(MIRROR ? min(q, s.lomin[p]) : max(q, s.lomin[p]));
        if (MIRROR ? lastfin > far : lastfin < far) { // no stage of this row starts from a layer the table has reached
            for (int g = lane; g <= M; g += 64) G[r * (M + 1) + g] = kNone;
            wave_sync();
            continue;
        }
        bool fin = false;
        const int trips = MIRROR ? far - p : p - far; // stages [x, p), x = p-1 .. far / [p, x), x = p+1 .. far
        for (int gt = 0; gt * 8 < M; ++gt) {
            const int g = gt * 8 + gi + 1;
            double acc = kNone;
            for (int dt = 0; dt <= gt; ++dt) {
                const int dd = dt * 8 + di + 1;
                const bool on = g <= M && dd <= g;
                // Every lane walks the row's whole reach (uniform trip count, loads without conditions),
                // in groups of four trips: the four table entries and the four stage times are read
                // before any of them is used (one wait per group instead of one per trip).
                if (!MIRROR) {
                    // a trip beyond the lane's own reach or GPU count reads a valid stage time and, from
                    // the table, the entry (row 0, one GPU), which is "impossible" in every table
                    const int reach = on ? s.lo[p * M + dd - 1] : p;
                    const int mine = p - max(q, reach); // trips of this lane
                    const int ddc = on ? dd : 1, gc = on ? g - dd : 0;
                    int to = (p * M + ddc - 1) * (L + 1) + p - 1, go = (p - 1 - q) * (M + 1) + gc;
                    for (int i = 0; i < trips; i += 4) { // stage [x, p), x = p - 1 - i; table row x - q
                        double tt[4], gv[4];
#pragma unroll
                        for (int j = 0; j < 4; ++j) tt[j] = a.tdp[to - j];
#pragma unroll
                        for (int j = 0; j < 4; ++j) gv[j] = G[i + j < mine ? go - j * (M + 1) : 1];
#pragma unroll
                        for (int j = 0; j < 4; ++j) acc = fmin(acc, gv[j] + (wt * tt[j] + add));
                        to -= 4; go -= 4 * (M + 1);
                    }
                } else {
                    // a lane without a pair walks the row of impossible stages; the others take every stage
                    // with t <= tau (t is not monotone along the walk, so the test is on the value)
                    const int row = on ? p * M + dd - 1 : (L + 1) * M, gc = on ? g - dd : 0;
                    int to = row * (L + 1) + p + 1, go = (q - p - 1) * (M + 1) + gc;
                    for (int i = 0; i < trips; i += 4) { // stage [p, x), x = p + 1 + i; table row q - x
                        double tt[4], gv[4];
#pragma unroll
                        for (int j = 0; j < 4; ++j) tt[j] = a.tds[to + j];
#pragma unroll
                        for (int j = 0; j < 4; ++j) gv[j] = G[go - j * (M + 1)];
#pragma unroll
                        for (int j = 0; j < 4; ++j) acc = fmin(acc, gv[j] + (wt * (tt[j] <= tau ? tt[j] : kNone) + add));
                        to += 4; go -= 4 * (M + 1);
                    }
                }
            }
            acc = min8(acc);
            if (di == 0 && g <= M) G[r * (M + 1) + g] = acc;
            fin = fin || acc < kNone;
        }
        if (lane == 0) G[r * (M + 1)] = kNone;
        if (__any(fin)) lastfin = p; // the same in every lane
        wave_sync();
    }
    // a whole node covering [q, p) (prefix) / [p, q) (suffix), and the partial covers next to the slowest stage
    for (int r = 1 + lane; r <= rows; r += 64) {
        const int p = MIRROR ? q - r : q + r;
        s.W[MIRROR ? widx(p, q, L) : widx(q, p, L)] = G[r * (M + 1) + M];
    }
    for (int g = 1 + lane; g < M; g += 64) s.GU[q * M + g] = G[rows * (M + 1) + g];
    wave_sync();
}

// Node after node, one step: OUT[c][g] from NP_c, and NP_{c+1} from NP_c (cur -> nxt).  NP_c[p]: c whole
// nodes cover [0, p) (prefix) / [p, L) (suffix).  Called by `nth` threads (whole waves), th = 0 .. nth-1.
template <bool MIRROR>
__device__ void node_step(const Args &a, const Lds &s, int e, int c, int cend, const double *cur, double *nxt,
                          double *OUT, int th, int nth) {
    const int L = a.L, M = a.M, h4 = th & 3;
    for (int i = th; i < M * 4; i += nth) { // four threads per g
        const int g = i >> 2;
        double m = kNone;
        if (g == 0) { if (h4 == 0) m = cur[e]; }
        else if (!MIRROR) for (int q = c + h4; q < e; q += 4) m = fmin(m, cur[q] + s.GU[q * M + g]); // c nodes cover at least c layers
        else              for (int q = e + 1 + h4; q <= L - c; q += 4) m = fmin(m, cur[q] + s.GU[q * M + g]);
        m = min4(m);
        if (h4 == 0) OUT[c * M + g] = m;
    }
    if (c + 1 < cend) {
        const int np = MIRROR ? L - e + 1 : e + 1; // layers of the side, origin included
        for (int i = th; i < ((np * 4 + 63) & ~63); i += nth) { // whole waves
            const int pi = i >> 2;
            double m = kNone;
            if (pi < np) {
                const int p = MIRROR ? L - pi : pi;
                if (!MIRROR) for (int q = c + h4; q < p; q += 4) m = fmin(m, cur[q] + s.W[widx(q, p, L)]);
                else         for (int q = p + 1 + h4; q <= L - c; q += 4) m = fmin(m, cur[q] + s.W[widx(p, q, L)]);
            }
            m = min4(m);
            if (h4 == 0 && pi < np) nxt[MIRROR ? L - pi : pi] = m;
        }
    }
}

__global__ void __launch_bounds__(1024) k_exact_lds(Args a) {
    HIP_DYNAMIC_SHARED(double, s_dyn)
    __shared__ unsigned s_next;
    if (*a.status != OOB_OK) return; // the same for every thread: nothing is computed from a bad profile
    const int L = a.L, M = a.M, count = a.n_max - a.n_min + 1, nw = blockDim.x >> 6;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    Lds s;
    double *p = s_dyn;
    s.W = p;    p += tri(L);
    s.GU = p;   p += (size_t)(L + 1) * M;
    s.NP = p;   p += 4 * (size_t)(L + 1);
    s.PU = p;   p += (size_t)a.n_max * M;
    s.SV = p;   p += (size_t)a.n_max * M;
    s.lo = (int *)p;    p += ((size_t)(L + 1) * M + 1) / 2;
    s.lomin = (int *)p; p += (size_t)(L + 1) / 2 + 1;
    s.bnd = p;  p += L;
    s.best = (unsigned long long *)p; p += count;
    s.G = p;
    // rows -kGPad .. -1 of a wave's one-node table stay "impossible": the walks run in groups of four
    // and may pass the table's first row
    double *G = s.G + (size_t)wave * (L + 1 + kGPad) * (M + 1) + kGPad * (M + 1);
    for (int g = lane; g < kGPad * (M + 1); g += 64) G[g - kGPad * (M + 1)] = kNone;
    const long long *bnd = (const long long *)a.prof.boundary_ns;
    for (int i = threadIdx.x; i < L; i += blockDim.x) s.bnd[i] = (double)bnd[i];
    for (int i = threadIdx.x; i < count; i += blockDim.x) s.best[i] = 0x7FF0000000000000ull;
    // weights of a stage before / after the slowest one and of the slowest one, as (t, tau) coefficients
    const double ptau = a.Nb > 0 ? 0.0 : 4.0, stau = a.Nb > 0 ? -1.0 : 3.0, mid = a.Nb > 0 ? (double)a.Nb : 4.0;
    const unsigned ncand = (unsigned)((long long)L * (L + 1) / 2 * M);
    // node-level phase: the first half of the waves takes the prefix side, the second half the suffix side
    const int nwp = (nw + 1) >> 1, mir = wave >= nwp && nw > 1;
    const int th = mir ? (int)threadIdx.x - nwp * 64 : (int)threadIdx.x, nth = nw > 1 ? (mir ? nw - nwp : nwp) * 64 : 64;
    for (;;) {
        __syncthreads(); // the previous candidate is done with LDS (and s_next has been read)
        if (threadIdx.x == 0) s_next = atomicAdd(a.counter, 1u);
        __syncthreads();
        const unsigned c = s_next;
        if (c >= ncand) break; // every wave of every workgroup gets here
        // candidate c -> (u, v, d): pairs u < v in row order, d fastest
        const int d = (int)(c % M) + 1;
        unsigned pr = c / M;
        int u = 0;
        while (pr >= (unsigned)(L - u)) { pr -= L - u; ++u; }
        const int v = u + 1 + (int)pr;
        const double tau = a.tds[((size_t)u * M + d - 1) * (L + 1) + v];
        if (!(tau < kNone)) continue; // the same for the whole workgroup
        // ---- reach of a stage into every layer 1..u and out of every layer v..L-1, per GPU count ----
        for (int i = threadIdx.x; i < (L + 1) * M; i += blockDim.x) {
            const int pl = i / M, dd = i % M + 1;
            int r = pl;
            if (pl >= 1 && pl <= u) r = side_reach<false>(a, s, pl, dd, tau);
            else if (pl >= v && pl < L) r = side_reach<true>(a, s, pl, dd, tau);
            s.lo[i] = r;
            s.GU[i] = kNone;
        }
        __syncthreads();
        for (int pl = threadIdx.x; pl <= L; pl += blockDim.x) {
            int m = s.lo[pl * M];
            if (pl <= u) for (int dd = 2; dd <= M; ++dd) m = min(m, s.lo[pl * M + dd - 1]);
            else         for (int dd = 2; dd <= M; ++dd) m = max(m, s.lo[pl * M + dd - 1]);
            s.lomin[pl] = m;
        }
        __syncthreads();
        // ---- phase 1: one-node tables, one start layer per wave at a time; the longest first, the two
        // sides in turn (prefix starts 0 .. u-1 have u, u-1, .. rows, suffix starts L .. v+1 have L-v, .. rows)
        {
            const int nP = u, nS = L - v, both = 2 * min(nP, nS);
            for (int item = wave; item < nP + nS; item += nw) {
                int side, idx;
                if (item < both) { side = item & 1; idx = item >> 1; }
                else { side = nS > nP; idx = item - (both >> 1); }
                if (!side) one_node_table<false>(a, s, u, idx, tau, 1.0, ptau * tau, G);
                else       one_node_table<true>(a, s, v, L - idx, tau, 2.0, stau * tau, G);
            }
        }
        __syncthreads();
        // ---- phase 2: node after node, both sides at once -----------------------------------------
        {
            // a node covers at least one layer: more whole nodes than a side has layers cover nothing
            const int cendP = min(a.n_max, u + 1), cendS = min(a.n_max, L - v + 1);
            double *curP = s.NP, *nxtP = s.NP + (L + 1), *curS = s.NP + 2 * (L + 1), *nxtS = s.NP + 3 * (L + 1);
            for (int pl = threadIdx.x; pl <= L; pl += blockDim.x) {
                curP[pl] = pl == 0 ? 0.0 : kNone;
                curS[pl] = pl == L ? 0.0 : kNone;
            }
            for (int i = threadIdx.x + cendP * M; i < a.n_max * M; i += blockDim.x) s.PU[i] = kNone;
            for (int i = threadIdx.x + cendS * M; i < a.n_max * M; i += blockDim.x) s.SV[i] = kNone;
            __syncthreads();
            const int cmax = max(cendP, cendS);
            for (int cc = 0; cc < cmax; ++cc) {
                if (nw > 1) {
                    if (!mir) { if (cc < cendP) node_step<false>(a, s, u, cc, cendP, curP, nxtP, s.PU, th, nth); }
                    else      { if (cc < cendS) node_step<true>(a, s, v, cc, cendS, curS, nxtS, s.SV, th, nth); }
                } else {
                    if (cc < cendP) node_step<false>(a, s, u, cc, cendP, curP, nxtP, s.PU, th, nth);
                    if (cc < cendS) node_step<true>(a, s, v, cc, cendS, curS, nxtS, s.SV, th, nth);
                }
                __syncthreads();
                double *tmp = curP; curP = nxtP; nxtP = tmp;
                tmp = curS; curS = nxtS; nxtS = tmp;
            }
        }
        // ---- the slowest stage at every place it fits, for every template whose stage limit cannot bind:
        // ca whole nodes and g GPUs before it, cb whole nodes and M - d - g GPUs after it, n = ca + cb + 1
        const int places = M - d + 1; // g = 0 .. M - d GPUs of its node before it
        for (int i = threadIdx.x; i < a.n_max * a.n_max; i += blockDim.x) {
            const int ca = i / a.n_max, cb = i % a.n_max, n = ca + cb + 1;
            if (n < a.n_min || n > a.n_max || (a.Nb > 0 && a.Nb < min(L, n * M))) continue;
            double m = kNone;
            for (int g = 0; g < places; ++g) m = fmin(m, s.PU[ca * M + g] + s.SV[cb * M + (M - d - g)]);
            m += mid * tau;
            if (m < kNone) atomicMin(&s.best[n - a.n_min], (unsigned long long)__double_as_longlong(m));
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < count; i += blockDim.x)
        if (s.best[i] != 0x7FF0000000000000ull) atomicMin(&a.best[i], s.best[i]);
}

// Results as int64: -1 where no pipeline exists, -2 (unstaged entry point) where the stage limit
// can bind, so that the minimum without it is not the answer.
__global__ void k_exact_finish(Args a, int from_double, int staged) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i > a.n_max - a.n_min) return;
    const int n = a.n_min + i;
    long long out;
    if (!staged && a.Nb > 0 && a.Nb < min(a.L, n * a.M)) out = -2;
    else if (from_double) { const double x = __longlong_as_double((long long)a.best[i]); out = x < kNone ? (long long)x : -1; }
    else out = (long long)a.best[i] >= kInf / 2 ? -1 : (long long)a.best[i];
    ((long long *)a.best)[i] = out;
}

// ---------------------------------------------------------------------------------------------
// The general path: tables in the workspace.
//   Pre[p][D][j] = least sum over sequences covering [0, p) on exactly the first D GPUs (with j stages), t < tau
//   Suf[p][E][j] = the same for [p, L) on exactly the last E GPUs, t <= tau
// STAGED = false: J = 1, the sums carry the weights of the cost; STAGED = true: plain sums of t, the
// stage counts choose the coefficient of tau at the end and obey j1 + 1 + j2 <= N_b.
// One workgroup takes one candidate slowest stage at a time (a grid-stride loop), walks the layers
// with two barriers per layer (the stage times into / out of the layer are staged in LDS), each
// thread owning (GPUs, stages) positions.
// ---------------------------------------------------------------------------------------------
template <bool STAGED>
__global__ void __launch_bounds__(kThreads) k_exact_flat(Args a) {
    HIP_DYNAMIC_SHARED(long long, s_flat) // [L * M] stage times into (or out of) the current layer, then [count] minima
    const int L = a.L, M = a.M, W = a.Dmax + 1, J = STAGED ? a.Smax + 1 : 1, count = a.n_max - a.n_min + 1;
    long long *s_col = s_flat, *s_best = s_flat + (size_t)L * M;
    const size_t plane = (size_t)W * J;
    long long *Pre = a.slots + (size_t)blockIdx.x * 2 * (L + 1) * plane, *Suf = Pre + (size_t)(L + 1) * plane;
    const long long *bnd = (const long long *)a.prof.boundary_ns;
    if (*a.status != OOB_OK) return;
    const long long ptau = STAGED ? 0 : (a.Nb > 0 ? 0 : 4), stau = STAGED ? 0 : (a.Nb > 0 ? -1 : 3);
    const long long wsuf = STAGED ? 1 : 2;
    for (int i = threadIdx.x; i < count; i += kThreads) s_best[i] = kInf;
    const long long ncand = (long long)L * (L + 1) / 2 * M;
    for (long long c = blockIdx.x; c < ncand; c += gridDim.x) {
        const int d = (int)(c % M) + 1;
        long long pr = c / M;
        int u = 0;
        while (pr >= L - u) { pr -= L - u; ++u; }
        const int v = u + 1 + (int)pr;
        const long long tau = a.t[((size_t)u * (L + 1) + v) * M + d - 1];
        if (tau < 0) continue;
        __syncthreads(); // the tables of the previous candidate are no longer read
        for (size_t i = threadIdx.x; i < plane; i += kThreads) Pre[i] = i == 0 ? 0 : kInf;
        for (int p = 1; p <= u; ++p) {
            __syncthreads();
            for (int i = threadIdx.x; i < p * M; i += kThreads) // times of the stages [q, p) on dd GPUs
                s_col[i] = a.t[((size_t)(i / M) * (L + 1) + p) * M + i % M];
            __syncthreads();
            for (size_t i = threadIdx.x; i < plane; i += kThreads) {
                const int D = (int)(i / J), j = (int)(i % J);
                long long m = kInf;
                if (!STAGED || j >= 1)
                    for (int dd = 1; dd <= M && dd <= D; ++dd) {
                        const int D0 = D - dd;
                        if (D0 % M + dd > M) continue; // would cross a node boundary
                        const size_t src = (size_t)D0 * J + (STAGED ? j - 1 : 0);
                        for (int q = p - 1; q >= 0; --q) { // [q, p) only gets slower and heavier as q goes down
                            const long long tt = s_col[q * M + dd - 1];
                            if (tt < 0 || tt >= tau) break;
                            const long long x = Pre[(size_t)q * plane + src] + tt + ptau * tau;
                            m = x < m ? x : m;
                        }
                    }
                Pre[(size_t)p * plane + i] = m;
            }
        }
        __syncthreads();
        for (size_t i = threadIdx.x; i < plane; i += kThreads) Suf[(size_t)L * plane + i] = i == 0 ? 0 : kInf;
        for (int p = L - 1; p >= v; --p) {
            __syncthreads();
            for (int i = threadIdx.x; i < (L - p) * M; i += kThreads) // times of the stages [p, p+1+i/M) on dd GPUs
                s_col[i] = a.t[((size_t)p * (L + 1) + p + 1 + i / M) * M + i % M];
            __syncthreads();
            for (size_t i = threadIdx.x; i < plane; i += kThreads) {
                const int E = (int)(i / J), j = (int)(i % J);
                long long m = kInf;
                if (!STAGED || j >= 1)
                    for (int dd = 1; dd <= M && dd <= E; ++dd) {
                        const int E0 = E - dd;
                        if (E0 % M + dd > M) continue;
                        const size_t src = (size_t)E0 * J + (STAGED ? j - 1 : 0);
                        // [p, w) as w goes up: impossible stays impossible and the time without the boundary
                        // term only grows, so those end the loop; a stage that is only too slow because of
                        // the boundary term of its last layer is skipped, not the rest of the run
                        for (int w = p + 1; w <= L; ++w) {
                            const long long tt = s_col[(w - p - 1) * M + dd - 1];
                            if (tt < 0) break;
                            if (tt > tau) {
                                if (w == L || tt - bnd[w - 1] > tau) break;
                                continue;
                            }
                            const long long x = Suf[(size_t)w * plane + src] + wsuf * tt + stau * tau;
                            m = x < m ? x : m;
                        }
                    }
                Suf[(size_t)p * plane + i] = m;
            }
        }
        __syncthreads();
        // the slowest stage at every place it fits, for every template
        for (size_t i = threadIdx.x; i < plane; i += kThreads) {
            const int D = (int)(i / J), j1 = (int)(i % J);
            if (D + d > a.Dmax) continue;
            if (D % M + d > M) continue;
            const long long pre = Pre[(size_t)u * plane + i];
            if (pre >= kInf / 2) continue;
            for (int n = a.n_min; n <= a.n_max; ++n) {
                const int E = n * M - D - d;
                if (E < 0) continue;
                if (!STAGED) {
                    if (a.Nb > 0 && a.Nb < min(L, n * M)) continue;
                    const long long suf = Suf[(size_t)v * plane + E];
                    if (suf >= kInf / 2) continue;
                    const long long tot = pre + (a.Nb > 0 ? (long long)a.Nb : 4ll) * tau + suf;
                    if (tot < s_best[n - a.n_min]) atomicMin((unsigned long long *)&s_best[n - a.n_min], (unsigned long long)tot);
                } else {
                    for (int j2 = 0; j1 + 1 + j2 <= a.Smax; ++j2) {
                        const long long suf = Suf[(size_t)v * plane + (size_t)E * J + j2];
                        if (suf >= kInf / 2) continue;
                        const long long coef = a.Nb > 0 ? (long long)a.Nb - j2 : 4ll * j1 + 4 + 3ll * j2;
                        const long long tot = pre + coef * tau + 2 * suf;
                        if (tot < s_best[n - a.n_min]) atomicMin((unsigned long long *)&s_best[n - a.n_min], (unsigned long long)tot);
                    }
                }
            }
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < count; i += kThreads)
        if (s_best[i] < kInf) atomicMin(&a.best[i], (unsigned long long)s_best[i]);
}

inline size_t slot_bytes(int L, int Dmax, int J) { return align_up(sizeof(long long) * 2 * (size_t)(L + 1) * (Dmax + 1) * J); }

} // namespace oob_exact

static bool exact_dims_ok(int L, int n_max, int M) {
    return L >= 1 && L <= OOB_EXACT_MAX_L && n_max >= 1 && M >= 1 && M <= OOB_MAX_GPUS &&
           (long long)n_max * M <= OOB_EXACT_MAX_GPUS;
}
static int exact_smax(int L, int n_max, int M, int Nb) {
    int s = L < n_max * M ? L : n_max * M;
    return Nb > 0 && Nb < s ? Nb : s;
}

extern "C" size_t oob_exact_workspace_size(int L, int n_max, int gpus_per_node) {
    using namespace oob_exact;
    if (!exact_dims_ok(L, n_max, gpus_per_node)) return 0;
    size_t n = head_bytes(L, gpus_per_node);
    if (lds_waves(L, gpus_per_node, n_max, n_max) == 0) // tables beyond LDS: the general path
        n += (size_t)kFlatSlots * slot_bytes(L, n_max * gpus_per_node, 1);
    return n;
}

extern "C" size_t oob_exact_staged_workspace_size(int L, int n_max, int gpus_per_node, int microbatches) {
    using namespace oob_exact;
    if (!exact_dims_ok(L, n_max, gpus_per_node) || microbatches < 0) return 0;
    const size_t slot = slot_bytes(L, n_max * gpus_per_node, exact_smax(L, n_max, gpus_per_node, microbatches) + 1);
    const size_t want = (size_t)1 << 30; // about a gigabyte of tables, at least 16 and at most kFlatSlots workgroups in flight
    size_t slots = want / slot;
    slots = slots < 16 ? 16 : slots > (size_t)kFlatSlots ? (size_t)kFlatSlots : slots;
    return head_bytes(L, gpus_per_node) + slots * slot;
}

static int exact_launch(const oob_profile *profile, int L, int n_min, int n_max, int M, int microbatches, int64_t mem_cap,
                        void *dev_workspace, size_t workspace_bytes, int64_t *best, int32_t *status, void *stream,
                        bool staged) {
    using namespace oob_exact;
    if (!profile || !profile->fwd_ns || !profile->bwd_ns || !profile->mem_bytes || !profile->boundary_ns) return OOB_EINVAL;
    if (!best || !status || !dev_workspace || ((uintptr_t)dev_workspace & 255) != 0) return OOB_EINVAL;
    if (n_min < 1 || n_min > n_max || mem_cap <= 0 || microbatches < 0 || !exact_dims_ok(L, n_max, M)) return OOB_EINVAL;
    const int count = n_max - n_min + 1, Dmax = n_max * M;
    Args a;
    a.prof = *profile; a.L = L; a.M = M; a.n_min = n_min; a.n_max = n_max; a.Nb = microbatches; a.Dmax = Dmax;
    a.Smax = exact_smax(L, n_max, M, microbatches);
    a.cap = mem_cap;
    char *ws = (char *)dev_workspace;
    a.counter = (unsigned *)ws;
    a.t = (long long *)(ws + 256);
    a.tds = (double *)(ws + 256 + align_up(8 * table_entries(L, M)));
    a.tdp = (double *)(ws + 256 + align_up(8 * table_entries(L, M)) + align_up(8 * dtable_entries(L, M)));
    a.slots = (long long *)(ws + head_bytes(L, M));
    a.best = (unsigned long long *)best; a.status = status;
    hipStream_t st = (hipStream_t)stream;
    const int nw = staged ? 0 : lds_waves(L, M, n_max, count);
    const int J = staged ? a.Smax + 1 : 1;
    size_t slots = 0;
    if (nw == 0) {
        if (workspace_bytes < head_bytes(L, M) + 16 * slot_bytes(L, Dmax, J)) return OOB_ECAPACITY;
        slots = (workspace_bytes - head_bytes(L, M)) / slot_bytes(L, Dmax, J);
        if (slots > (size_t)kFlatSlots) slots = kFlatSlots;
    } else if (workspace_bytes < head_bytes(L, M)) return OOB_ECAPACITY;
    a.limit = nw ? kDoubleExact : kInf;
    hipLaunchKernelGGL(k_exact_init, dim3(1), dim3(kThreads), 0, st, a);
    hipLaunchKernelGGL(k_exact_fill, dim3(64), dim3(256), 0, st, a);
    hipLaunchKernelGGL(k_exact_stages, dim3((L * M + 63) / 64), dim3(64), 0, st, a);
    const long long ncand = (long long)L * (L + 1) / 2 * M;
    if (nw) {
        const size_t lds = lds_bytes(L, M, n_max, count, nw);
        if (lds > 64 * 1024 &&
            hipFuncSetAttribute((const void *)k_exact_lds, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
            return OOB_EHIP;
        const unsigned grid = (unsigned)(ncand < 512 ? ncand : 512); // two rounds of workgroups per compute unit; a counter hands out the work
        hipLaunchKernelGGL(k_exact_lds, dim3(grid), dim3(nw * 64), lds, st, a);
    } else {
        const unsigned grid = (unsigned)(ncand < (long long)slots ? ncand : (long long)slots);
        const size_t lds = sizeof(long long) * ((size_t)L * M + count);
        if (staged) hipLaunchKernelGGL(k_exact_flat<true>, dim3(grid), dim3(kThreads), lds, st, a);
        else        hipLaunchKernelGGL(k_exact_flat<false>, dim3(grid), dim3(kThreads), lds, st, a);
    }
    hipLaunchKernelGGL(k_exact_finish, dim3((count + 63) / 64), dim3(64), 0, st, a, nw ? 1 : 0, staged ? 1 : 0);
    return hipGetLastError() == hipSuccess ? OOB_OK : OOB_EHIP;
}

extern "C" int oob_exact_minimum(const oob_profile *profile, int L, int n_min, int n_max, int gpus_per_node,
                                 int microbatches, int64_t mem_cap, void *dev_workspace, size_t workspace_bytes,
                                 int64_t *best, int32_t *status, void *stream) {
    return exact_launch(profile, L, n_min, n_max, gpus_per_node, microbatches, mem_cap, dev_workspace, workspace_bytes,
                        best, status, stream, false);
}

extern "C" int oob_exact_minimum_staged(const oob_profile *profile, int L, int n_min, int n_max, int gpus_per_node,
                                        int microbatches, int64_t mem_cap, void *dev_workspace, size_t workspace_bytes,
                                        int64_t *best, int32_t *status, void *stream) {
    return exact_launch(profile, L, n_min, n_max, gpus_per_node, microbatches, mem_cap, dev_workspace, workspace_bytes,
                        best, status, stream, true);
}
