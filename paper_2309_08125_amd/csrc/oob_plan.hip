// MI355X (gfx950) pipeline-template planner: kernels and host driver behind the C ABI of
// include/oob_plan.h.  Method: Section 4.1 of the Oobleck paper (node specification 4.1.1,
// GPU-stage mapping 4.1.2 with Eq. 1-4, coverage theorem of Appendix A).
//
// Arithmetic.  Inputs and outputs are int64.  Inside the tables every time is held as an
// IEEE double: gfx950 issues 64-bit floating add / min / compare at full rate (one VALU
// instruction each) while a 64-bit integer add or compare takes two or more, and doubles are
// exact for integers below 2^53.  The set-up kernel proves the bound (every quantity the
// recursion can form stays below 2^52 ns, about 52 days) or reports OOB_EOVERFLOW, so the
// results are bit-identical to int64 arithmetic in any evaluation order.
//
// What a state stores.  With r = S' - s and children A = (s, u, k, left set),
// B = (r, k, v, right set), Eq. 1-3 give the candidate's total
//     slowest stage in A (A.tmax >= B.tmax):  T = (A.T + cl * A.tmax) + 2 * B.T1
//     slowest stage in B:                     T = A.T1 + (B.T + cr * B.tmax)
// where X.T is the child's own total under its own stage count, and (cl, cr) = (-r, 0) when
// N_b is the caller's microbatch count or (3r, 4s) when N_b = 4 S' per state.  So the hot
// loop needs only (T, T1, tmax) per child: 2 adds, 1 compare, 2 selects, 1 min per candidate.
// T3 and k* are carried per state for the output only.
//
// One level S' = split kernels, then a select kernel.
//   k_split_key  per (block of the (u,v) plane, segment of its split points k, split s, group of
//            target device sets): the minimum over (k, m) of Eq. 1-3 per state as a key
//            total * 2^kbits + k, merged into the level's key array (described at the kernel).
//            k_split is the variant without keys for shapes beyond its LDS classes.
//   k_select / k_select8  per state: first s with the smallest key, then the first m at that
//            (s, k) whose candidate equals it -- the smallest (T, s, k, m) -- and the record.
// Before level 1 one launch (k_prepare) scans and validates the profile, lays out the tables, lists the
// tasks of every level and clears the keys; after the last level k_pick chooses the stage count of
// every template size, k_backtrack expands the stages, k_coverage does Section 4.1.1's node specification.
#include <hip/hip_runtime.h>

#include <mutex>
#include <type_traits>
#include <algorithm>
#include <vector>
#include <math.h>
#include <new>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "oob_layout.h"
#include "oob_plan.h"

namespace oob {

constexpr double kNone = __builtin_huge_val(); // total of a state that does not exist
constexpr long long kExactBound = 1LL << 52;
constexpr int kInternalError = -5;             // status: a state's minimum was not re-found

struct Rec { double T, T1, tmax, T3; };        // 32 bytes, one per (table, u, v)

// Device view of the workspace.
struct Tables {
    Shape sh;
    int NB;               // blocks per side of the (u, v) plane
    int coff;             // column shift of the plane: v sits in block column (v + coff) / 8
    int tab_recs;         // records per table = tri_blocks(NB) * 64
    long long *lvl_tab;   // [Smax+2] index of the first table of level S'
    long long *PT;        // [(M+1)*(L+1)] prefix sums of F+B for d GPUs (row d)
    int *PF;              // [(M+1)*(L+1)] prefix counts of forbidden entries
    long long *PM;        // [L+1] prefix sums of bytes
    Rec *rec;             // [tables * tab_recs]
    int *kstar, *choice;  // [tables * tab_recs]
    double *partT;        // [(S'-1) * deltas * tiles * 64] per-split minima of the current level
    unsigned long long *partKey; // the same memory: keys total * 2^kbits + k (keyed kernel)
    int *partK;           // same shape: first k reaching the minimum
    int *stack;           // backtracking stacks / coverage ring
    int2 *seg_tab;        // per level: (tile index, ub | vb << 8 | segment << 16) of every split task
    int seg_stride;       // entries reserved per level in seg_tab (level S' starts at (S'-2) * seg_stride)
    int *flags;           // [0] 1: (total, k) keys fit a double and k_split_key runs
                          // [1] 1: the host chose the plain split kernel k_split for this job (then [0] = 0)
                          // [0] = [1] = 0: k_select evaluates every candidate itself
    int *status;
};

__device__ __forceinline__ long long rec_index(const Tables &t, int S, int delta, int u, int v) {
    const long long tab = t.lvl_tab[S] + (delta - dlo_of(S, t.sh.M));
    return tab * t.tab_recs + rec_off(u, v, t.coff, t.NB);
}
// First record of block (ub, vb) of that table.
__device__ __forceinline__ long long rec_block(const Tables &t, int S, int delta, int ub, int vb) {
    const long long tab = t.lvl_tab[S] + (delta - dlo_of(S, t.sh.M));
    return tab * t.tab_recs + (long long)tri_index(ub, vb, t.NB) * 64;
}

// ---------------------------------------------------------------------------------------
// Set-up: prefix sums (Eq. 4's sums become differences), input validation, level offsets.
// One workgroup of four waves: two of them scan the profile rows of d GPUs, 64 entries at a time (sums
// saturate, so that no input can overflow them; a saturated sum is reported, not used); one wave
// scans the bytes and the boundary terms, one lays out the levels.
// ---------------------------------------------------------------------------------------
constexpr int kSetupThreads = 256; // a larger workgroup waits long for a place on a GPU that other jobs of a batch keep busy

// Inclusive scan over the lanes of min(a + b, cap) for values in [0, cap], cap <= 2^62.
__device__ __forceinline__ unsigned long long scan_sat(unsigned long long x, unsigned long long cap, int lane) {
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const unsigned long long y = __shfl_up(x, d, 64);
        if (lane >= d) { x += y; if (x > cap) x = cap; }
    }
    return x;
}
__device__ __forceinline__ int scan_int(int x, int lane) {
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int y = __shfl_up(x, d, 64);
        if (lane >= d) x += y;
    }
    return x;
}

__device__ void setup_body(const Tables &t, const oob_profile &prof, int force_plain) {
    const int L = t.sh.L, M = t.sh.M, W = L + 1;
    __shared__ long long s_worst[OOB_MAX_GPUS + 1];
    __shared__ int s_bad;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    if (threadIdx.x == 0) s_bad = 0;
    __syncthreads();
    const unsigned long long capT = (unsigned long long)kExactBound, capM = (unsigned long long)OOB_FORBIDDEN;
    int bad = 0;
    for (int d = 1 + wave; d <= M && wave < nw - 2; d += nw - 2) { // row of d GPUs
        unsigned long long carry = 0;
        int fcarry = 0;
        if (lane == 0) { t.PT[d * W] = 0; t.PF[d * W] = 0; }
        for (int l0 = 0; l0 < L; l0 += 64) {
            const int l = l0 + lane;
            const bool in = l < L;
            const long long F = in ? prof.fwd_ns[(size_t)l * M + d - 1] : 0, B = in ? prof.bwd_ns[(size_t)l * M + d - 1] : 0;
            const bool neg = F < 0 || B < 0;
            const bool fb = F >= OOB_FORBIDDEN || B >= OOB_FORBIDDEN;
            const bool big = !neg && !fb && (F >= kExactBound || B >= kExactBound);
            if (neg) bad = imax(bad, 1);
            if (big) bad = imax(bad, 2);
            unsigned long long x = (neg || fb || big) ? 0ull : (unsigned long long)(F + B);
            if (x > capT) x = capT;
            x = scan_sat(x, capT, lane) + carry;
            if (x > capT) x = capT;
            const int c = scan_int(fb ? 1 : 0, lane) + fcarry;
            if (in) { t.PT[d * W + l + 1] = (long long)x; t.PF[d * W + l + 1] = c; }
            carry = __shfl(x, 63, 64);
            fcarry = __shfl(c, 63, 64);
        }
        if (carry >= capT) bad = imax(bad, 2);
        if (lane == 0) s_worst[d] = (long long)carry;
    }
    if (wave == nw - 2) { // bytes and boundary terms
        unsigned long long cm = 0, cx = 0;
        if (lane == 0) t.PM[0] = 0;
        for (int l0 = 0; l0 < L; l0 += 64) {
            const int l = l0 + lane;
            const bool in = l < L;
            const long long mb = in ? prof.mem_bytes[l] : 0, xb = in ? prof.boundary_ns[l] : 0;
            const bool badm = mb < 0 || mb >= OOB_FORBIDDEN;
            if (badm || xb < 0) bad = imax(bad, 1);
            if (xb >= kExactBound) bad = imax(bad, 2);
            unsigned long long m = badm ? 0ull : (unsigned long long)mb;
            m = scan_sat(m, capM, lane) + cm;
            if (m > capM) m = capM;
            unsigned long long x = (xb < 0 || xb >= kExactBound) ? 0ull : (unsigned long long)xb;
            x = scan_sat(x, capT, lane) + cx;
            if (x > capT) x = capT;
            if (in) t.PM[l + 1] = (long long)m;
            cm = __shfl(m, 63, 64);
            cx = __shfl(x, 63, 64);
        }
        if (cm >= capM) bad = imax(bad, 1);
        if (cx >= capT) bad = imax(bad, 2);
        if (lane == 0) s_worst[0] = (long long)cx;
    }
    if (bad) atomicMax(&s_bad, bad);
    if (threadIdx.x == blockDim.x - 1) { // level offsets
        long long tab = 0;
        for (int S = 1; S <= t.sh.Smax + 1; ++S) {
            t.lvl_tab[S] = tab;
            const int nd = dhi_of(S, M, t.sh.n_max) - dlo_of(S, M) + 1;
            if (S <= t.sh.Smax && nd > 0) tab += nd;
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
            // a total and a split point k <= L fit one double as total * 2^kbits + k
            t.flags[0] = !force_plain && worst < (kExactBound >> key_bits(L)) / mult;
        }
        if (st != OOB_OK) t.flags[0] = 0;
        t.flags[1] = force_plain;
        *t.status = st;
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
// Level 1 ("Conquer", Eq. 4): grid (block of the plane, delta), one lane per (u, v).
// ---------------------------------------------------------------------------------------
__global__ void __launch_bounds__(64) k_level1(Tables t, const long long *X) {
    const int L = t.sh.L, M = t.sh.M;
    int ub, vb;
    tile_decode(L, 1, blockIdx.x, &ub, &vb);
    const int delta = blockIdx.y, u = ub * 8 + (threadIdx.x >> 3), v = vb * 8 + (threadIdx.x & 7) - t.coff;
    Rec r = {kNone, kNone, 0.0, 0.0};
    if (u < L && v <= L && v - u >= 1) { // (v < 0 in the first block column: no state)
        const int d = delta < M - 1 ? delta + 1 : M;
        long long st;
        if (stage_time(t, X, u, v, d, &st)) {
            const double nb = t.sh.Nb > 0 ? (double)t.sh.Nb : 4.0;
            r.T1 = r.tmax = r.T3 = (double)st;
            r.T = r.T1 + (nb - 2.0) * r.tmax + r.T3; // Eq. 2 with S' = 1, k* = 0
        }
    }
    const long long o = rec_block(t, 1, delta, ub, vb) + threadIdx.x;
    t.rec[o] = r;
    t.kstar[o] = 0;
    t.choice[o] = 0;
}

// ---------------------------------------------------------------------------------------
// Levels S' >= 2 ("Divide", Eq. 1-3), first kernel: per (s, state) the minimum over (k, m).
//   grid.x  block (ub, vb) of the plane      grid.y  s - 1      grid.z  group of 8*waves sets
//   fam     0: targets inside one node (units = GPUs), 1: whole-node targets (units = nodes)
// PC = k values staged per pass.
// ---------------------------------------------------------------------------------------
template <int PC>
__global__ void __launch_bounds__(512) k_split(Tables t, int Sp, int fam, int NT, int NAall) {
    HIP_DYNAMIC_SHARED(double2, s_pair) // [ntab][PC][8] (x, y) pairs, then double tmax[ntab][PC][8]
    if (t.flags[1] == 0) return;        // only when the host chose this kernel (it then launches no other)
    const int L = t.sh.L, M = t.sh.M, n_max = t.sh.n_max;
    const int s = blockIdx.y + 1, r = Sp - s;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    const int ul = lane >> 3, vl = lane & 7;
    int ub, vb;
    tile_decode(L, Sp, blockIdx.x, &ub, &vb);
    const int fam_base = fam ? M - 2 : -1;
    int t_lo, t_hi;
    target_units(fam, Sp, M, n_max, &t_lo, &t_hi);
    const int a_wg0 = t_lo + blockIdx.z * nw * 8, a_wg1 = imin(t_hi, a_wg0 + nw * 8 - 1);
    int A_lo, A_hi, B_lo, B_hi;
    child_units(fam, s, M, n_max, &A_lo, &A_hi);
    child_units(fam, r, M, n_max, &B_lo, &B_hi);
    // left / right unit counts some target of this workgroup pairs up
    const int mA0 = imax(A_lo, a_wg0 - B_hi), mA1 = imin(A_hi, a_wg1 - B_lo);
    const int mB0 = imax(B_lo, a_wg0 - A_hi), mB1 = imin(B_hi, a_wg1 - A_lo);
    const int kmin = ub * 8 + s, kmax = tile_vmax(L, vb) - r;
    const bool work = mA0 <= mA1 && mB0 <= mB1 && kmin <= kmax;
    const int nA = work ? mA1 - mA0 + 1 : 0, nB = work ? mB1 - mB0 + 1 : 0, dummy = nA + nB;
    constexpr int TS = PC * 8;
    double *s_tm = (double *)(s_pair + (size_t)(dummy + 1) * TS);

    // this wave's targets a0..a0+7 and the left unit counts they use
    const int a0 = a_wg0 + wave * 8, a1 = imin(a_wg1, a0 + 7);
    const int mw0 = imax(mA0, a0 - B_hi), mw1 = imin(mA1, a1 - B_lo);
    const bool wave_work = work && a0 <= a_wg1 && mw0 <= mw1;

    double best[8];
    int bestk[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) { best[q] = kNone; bestk[q] = 0; }

    if (work) {
        for (int e = threadIdx.x; e < TS; e += blockDim.x) { // the "no such table" slot
            s_pair[dummy * TS + e] = make_double2(kNone, kNone);
            s_tm[dummy * TS + e] = 0.0;
        }
        const double cl = t.sh.Nb > 0 ? -(double)r : 3.0 * r, cr = t.sh.Nb > 0 ? 0.0 : 4.0 * s;
        const long long tabA = t.lvl_tab[s] - dlo_of(s, M) + fam_base, tabB = t.lvl_tab[r] - dlo_of(r, M) + fam_base;
        const int fillA = nA * TS, fill = (nA + nB) * TS;
        for (int kc = (kmin / PC) * PC; kc <= kmax; kc += PC) {
            __syncthreads(); // previous pass fully consumed
            for (int e = threadIdx.x; e < fill; e += blockDim.x) {
                if (e < fillA) {       // left child (s, u, k, m): row u of block (ub, k/8)
                    const int tab = e / TS, rem = e - tab * TS, u_l = rem / PC, k_l = rem - u_l * PC;
                    const int k = kc + k_l;
                    const Rec a = t.rec[(tabA + mA0 + tab) * t.tab_recs + (long long)tri_index(ub, (k + t.coff) >> 3, t.NB) * 64 +
                                        (u_l << 3) + ((k + t.coff) & 7)];
                    const int o = (tab * PC + k_l) * 8 + u_l;
                    s_pair[o] = make_double2(a.T + cl * a.tmax, a.T1);
                    s_tm[o] = a.tmax;
                } else {               // right child (r, k, v, m'): row k of block (k/8, vb)
                    const int e2 = e - fillA, tab = e2 / TS, rem = e2 - tab * TS, k_l = rem >> 3, v_l = rem & 7;
                    const int k = kc + k_l;
                    const Rec b = t.rec[(tabB + mB0 + tab) * t.tab_recs + (long long)tri_index(k >> 3, vb, t.NB) * 64 +
                                        ((k & 7) << 3) + v_l];
                    const int o = ((nA + tab) * PC + k_l) * 8 + v_l;
                    s_pair[o] = make_double2(2.0 * b.T1, b.T + cr * b.tmax);
                    s_tm[o] = b.tmax;
                }
            }
            __syncthreads();
            if (!wave_work) continue;
#pragma unroll 1
            for (int kl = 0; kl < PC; ++kl) {
                const int k = kc + kl;
                if (k < kmin || k > kmax) continue;
                double cur[8];
#pragma unroll
                for (int q = 0; q < 8; ++q) cur[q] = kNone;
#pragma unroll 1
                for (int mm = mw0; mm <= mw1; mm += 8) {
                    double apa[8], at1[8], atm[8], bb2[15], bbt[15], btm[15];
#pragma unroll
                    for (int qm = 0; qm < 8; ++qm) {
                        const int m = mm + qm;
                        const int tab = m <= mA1 ? m - mA0 : dummy;
                        const int o = (tab * PC + kl) * 8 + ul;
                        const double2 p = s_pair[o];
                        apa[qm] = p.x; at1[qm] = p.y; atm[qm] = s_tm[o];
                    }
#pragma unroll
                    for (int d = 0; d < 15; ++d) {
                        const int mp = a0 - mm - 7 + d; // m' = (a0 + qa) - (mm + qm), d = qa - qm + 7
                        const int tab = (mp >= mB0 && mp <= mB1) ? nA + mp - mB0 : dummy;
                        const int o = (tab * PC + kl) * 8 + vl;
                        const double2 p = s_pair[o];
                        bb2[d] = p.x; bbt[d] = p.y; btm[d] = s_tm[o];
                    }
#pragma unroll
                    for (int qm = 0; qm < 8; ++qm)
#pragma unroll
                        for (int qa = 0; qa < 8; ++qa) {
                            const int d = qa - qm + 7;
                            const double T = atm[qm] >= btm[d] ? apa[qm] + bb2[d] : at1[qm] + bbt[d];
                            cur[qa] = fmin(cur[qa], T);
                        }
                }
#pragma unroll
                for (int q = 0; q < 8; ++q) { // first k that reaches the minimum
                    const bool lt = cur[q] < best[q];
                    best[q] = lt ? cur[q] : best[q];
                    bestk[q] = lt ? k : bestk[q];
                }
            }
        }
    }
    if (a0 <= a_wg1) {
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            if (a0 + q > a_wg1) break;
            const int aidx = fam_base + a0 + q - dlo_of(Sp, M);
            const long long slot = ((long long)(s - 1) * NAall + aidx) * NT + blockIdx.x;
            t.partT[slot * 64 + lane] = best[q];
            t.partK[slot * 64 + lane] = bestk[q];
        }
    }
}

// ---------------------------------------------------------------------------------------
// Levels S' >= 2, first kernel, keyed variant (runs when flags[0] = 1).
//
// Same result as k_split, different mapping.  A workgroup owns (block of the plane, segment of
// its split points, s) and a group of up to kKeyTargets target sets; per split point it stages
// the records of both children for every unit count it needs in LDS.  Work items are (k, block
// of eight unit counts of one child); the waves take them round robin.  An item keeps those
// eight records in registers and streams the other child: a step forms eight candidates, which
// belong to eight consecutive targets.  The eight running minima rotate: after a step the
// minimum of the lowest target is complete for this item and is merged into the workgroup's
// LDS table acc[a][lane] with an integer atomic min on the bits of key = total * 2^kbits + k
// (non-negative doubles order like their bit patterns).  The key makes the merge order-free
// and yields, per (s, state), the smallest total and the first k reaching it at once.
// ---------------------------------------------------------------------------------------
constexpr int kKeyTargets = 64;
constexpr int kFillBatch = 3;      // records a thread has in flight while staging: three waves per SIMD
constexpr int kFillBatchSmall = 2; // the same for launches whose LDS admits four workgroups per compute unit

// Workgroup x of a launch of n -> position in the task list (handle option OOB_OPT_XCD_ORDER only).  The hardware
// deals consecutive workgroups out to the 8 XCDs in turn; this hands every XCD one contiguous
// stretch of the list instead (workgroups x, x + 8, x + 16, ... walk it in order), so that tasks
// that share records meet in one L2.  A bijection on 0..n-1 for any n.  Measured on the headline
// workload: 29 % fewer bytes fetched from HBM, but 2 % more time (the stretches are not equally
// heavy and the kernel is bound by the vector ALUs), hence off by default.
__device__ __forceinline__ int xcd_chunked(int x, int n) {
    const int c = x & 7, i = x >> 3, q = n >> 3, rem = n & 7;
    return c * q + imin(c, rem) + i;
}

// The (m, m') pairs of a split form a rectangle; an item keeps eight records of one side in
// registers (the STATIONARY side, cut into blocks of eight unit counts, the last one padded) and
// streams the other side.  Which child is stationary is chosen per workgroup so that the padding
// is smaller (it is the same work either way).  Staging order for split point k:
// [streaming tables][lane index], then [stationary tables, padded][lane index]; the lane index
// is u for records of the left child and v for records of the right child.
struct Stage {
    const Rec *recY, *recS; // first record of the table of unit count 0 of the streaming / stationary side
    int tab_recs, NB, coff, ub, vb, nS, fillY, fill;
    int y_is_left;          // 1: left child streams, right child stationary; 0: the other way round
    double cl, cr;
};
struct Rec24 { double2 a; double tm; }; // (T, T1), tmax: the 24 bytes of a record the splits need

// Where the records of split point k sit inside a table: the left child (s, u, k, m) is row u of
// block (ub, k/8), column k; the right child (r, k, v, m') is row k of block (k/8, vb), column v.
// Scalar work, once per split point; per staged record only a 32-bit offset is left to form
// (tables of one side x records of a table x 32 bytes stays below 2^32).
struct StagePoint { const Rec *py, *ps; int shY, shS; };
__device__ __forceinline__ StagePoint stage_point(const Stage &g, int k) {
    const int ck = k + g.coff; // column of split point k in the left child's table
    const int offL = tri_index(g.ub, ck >> 3, g.NB) * 64 + (ck & 7), offR = tri_index(k >> 3, g.vb, g.NB) * 64 + ((k & 7) << 3);
    StagePoint sp;
    sp.py = g.recY + (g.y_is_left ? offL : offR);
    sp.ps = g.recS + (g.y_is_left ? offR : offL);
    sp.shY = g.y_is_left ? 3 : 0; // the lane index is a row of the block for left records, a column for right ones
    sp.shS = g.y_is_left ? 0 : 3;
    return sp;
}
__device__ __forceinline__ Rec24 stage_load(const Stage &g, const StagePoint &sp, int e) {
    Rec24 rc = {make_double2(kNone, kNone), 0.0};
    const bool stream = e < g.fillY;
    const int e2 = stream ? e : e - g.fillY, tab = e2 >> 3, idx = e2 & 7;
    if (e < g.fill && (stream || tab < g.nS)) {
        const unsigned off = (__umul24((unsigned)tab, (unsigned)g.tab_recs) + ((unsigned)idx << (stream ? sp.shY : sp.shS))) << 5;
        const Rec *p = (const Rec *)((const char *)(stream ? sp.py : sp.ps) + off);
        rc.a = *(const double2 *)p;
        rc.tm = p->tmax;
    }
    return rc;
}
// LDS order = staging order; values pre-combined with the level's coefficients: left records as
// (T + cl tmax, T1), right records as (2 T1, T + cr tmax).  The slowest-stage test of Eq. 3 is
// "left tmax >= right tmax"; the step loop always tests "streaming >= stationary", so when the
// right child streams both tmax are stored negated.
__device__ __forceinline__ void stage_store(const Stage &g, double2 *pair, double *tm, int e, const Rec24 &rc) {
    if (e >= g.fill) return;
    const bool left = (e < g.fillY) == (g.y_is_left != 0);
    pair[e] = left ? make_double2(rc.a.x + g.cl * rc.tm, rc.a.y) : make_double2(2.0 * rc.a.y, rc.a.x + g.cr * rc.tm);
    tm[e] = g.y_is_left ? rc.tm : -rc.tm;
}

// floor(x / d) for 0 <= x < 10000 and 1 <= d <= 4 without the division sequence (x 21846 >> 16 is
// exact for thirds in that range).
__device__ __forceinline__ int div_small(int x, int d) {
    return d == 1 ? x : d == 2 ? x >> 1 : d == 4 ? x >> 2 : (x * 21846) >> 16;
}

// Candidate slots an assignment of roles executes: per block of eight stationary unit counts the
// streaming range that pairs with it (targets a0..a1), times eight.
__host__ __device__ __forceinline__ int role_cost(int y0, int y1, int q0, int q1, int a0, int a1) {
    int c = 0;
    for (int qb = q0; qb <= q1; qb += 8) {
        const int lo = imax(y0, a0 - (qb + 7)), hi = imin(y1, a1 - qb);
        if (lo <= hi) c += hi - lo + 1;
    }
    return c;
}

// One split point per pass, one LDS buffer: while the waves work on k, every thread has the
// records of k+1 in flight from HBM/L2 and drops them into the buffer between the two barriers
// of the pass (NBUF = 2: two buffers and one barrier; needs more LDS, measured slower).
// FB = kFillBatch: 167 vector registers, three waves per SIMD.  FB = kFillBatchSmall: launch bounds hold
// the kernel to 128 registers (four waves per SIMD, for launches whose LDS admits a fourth workgroup
// per compute unit) at the price of 24 bytes of spills per lane in the per-pass code, none in the step
// loop; records beyond FB per thread are fetched between the barriers.  Measured on the headline
// workload: nothing in flight 9.78 ms, one record 9.84 ms, two 9.64 ms for the levels.
template <int NTAB, int NBUF, int FB>
__global__ void __launch_bounds__(256, FB == kFillBatch ? 1 : 4) k_split_key(Tables t, int Sp, int fam0, int gz, int NT, int NAall, int halves,
                                                   int s0, int sstep) {
    // Separate arrays (the staged records static, the key table the launch's dynamic LDS, sized by
    // its target count): the compiler then knows that the key merges (atomics on s_acc) never touch
    // the staged records, and keeps the reads of the next step ahead of them.
    __shared__ double2 s_pair[NBUF][NTAB * 8]; // [buffer][staging order]: pre-combined pairs
    __shared__ double s_tm[NBUF][NTAB * 8];    // tmax (negated when the right child streams)
    HIP_DYNAMIC_SHARED(unsigned long long, s_acc)       // [(na + 2) * 64] keys, rows 1..na (sized by the launch)
    if (t.flags[0] == 0) return;        // keys do not fit: k_select evaluates the candidates itself
    const int L = t.sh.L, M = t.sh.M, n_max = t.sh.n_max;
    const int s = s0 + blockIdx.y * sstep, r = Sp - s; // a launch covers the splits s0, s0 + sstep, ...
    // the wave index is the same in all lanes: say so, and everything derived from it (work item,
    // m range, key row) is scalar arithmetic and scalar branches
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), nw = blockDim.x >> 6;
    const int2 sg = t.seg_tab[(long long)(Sp - 2) * t.seg_stride + ((halves & 8) ? xcd_chunked(blockIdx.x, gridDim.x) : (int)blockIdx.x)]; // x: tile index, y: ub | vb << 8 | seg << 16
    const int tile = sg.x, ub = sg.y & 255, vb = (sg.y >> 8) & 255, seg = sg.y >> 16;
    // the first gz target groups of the launch belong to family fam0, the rest (a launch that covers
    // both families of a low level) to the whole-node family
    const int fam = (int)blockIdx.z < gz ? fam0 : 1, zg = (int)blockIdx.z < gz ? (int)blockIdx.z : (int)blockIdx.z - gz;
    const int fam_base = fam ? M - 2 : -1;
    int t_lo, t_hi;
    target_units(fam, Sp, M, n_max, &t_lo, &t_hi);
    const int a_g0 = t_lo + zg * kKeyTargets, a_g1 = imin(t_hi, a_g0 + kKeyTargets - 1);
    const int na = a_g1 - a_g0 + 1;
    int A_lo, A_hi, B_lo, B_hi;
    child_units(fam, s, M, n_max, &A_lo, &A_hi);
    child_units(fam, r, M, n_max, &B_lo, &B_hi);
    const int mA0 = imax(A_lo, a_g0 - B_hi), mA1 = imin(A_hi, a_g1 - B_lo);
    const int mB0 = imax(B_lo, a_g0 - A_hi), mB1 = imin(B_hi, a_g1 - A_lo);
    // this workgroup's segment of the split points of the block
    const int vmax = tile_vmax(L, vb); // last layer position of the block's columns (never beyond L)
    int kofs, klen;
    {
        const int kr = tile_krange(L, Sp, ub, vb);
        seg_span(kr, seg_n(kr, seg_target(L, Sp)), seg, &kofs, &klen);
    }
    const int kmin = ub * 8 + s + kofs, kmax = imin(vmax - r, kmin + klen - 1);
    if (!(mA0 <= mA1 && mB0 <= mB1 && kmin <= kmax)) return; // nothing to merge
    // roles: the left child streams (and the right one is stationary) unless the other way pads less
    const bool y_left = role_cost(mA0, mA1, mB0, mB1, a_g0, a_g1) <= role_cost(mB0, mB1, mA0, mA1, a_g0, a_g1);
    const int yM0 = y_left ? mA0 : mB0, yM1 = y_left ? mA1 : mB1; // streaming unit counts
    const int qM0 = y_left ? mB0 : mA0, qM1 = y_left ? mB1 : mA1; // stationary unit counts
    const int nY = yM1 - yM0 + 1, nS = qM1 - qM0 + 1, nmb = cdiv(nS, 8);
    const int fillY = nY * 8, TS = fillY + nmb * 64;
    const unsigned long long kNoneBits = 0x7FF0000000000000ull;
    const double KS = (double)(1 << key_bits(L));

    Stage g;
    const long long tabA = t.lvl_tab[s] - dlo_of(s, M) + fam_base, tabB = t.lvl_tab[r] - dlo_of(r, M) + fam_base;
    g.recY = t.rec + (y_left ? tabA + mA0 : tabB + mB0) * t.tab_recs;
    g.recS = t.rec + (y_left ? tabB + mB0 : tabA + mA0) * t.tab_recs;
    g.tab_recs = t.tab_recs; g.NB = t.NB; g.coff = t.coff; g.ub = ub; g.vb = vb; g.nS = nS;
    g.fillY = fillY; g.fill = TS; g.y_is_left = y_left;
    g.cl = t.sh.Nb > 0 ? -(double)r : 3.0 * r;
    g.cr = t.sh.Nb > 0 ? 0.0 : 4.0 * s;

    // rows 1..na are the targets; rows 0 and na+1 swallow the minima of targets outside the group
    for (int e = threadIdx.x; e < (na + 2) * 64; e += blockDim.x) s_acc[e] = kNoneBits;
    Rec24 pre[FB ? FB : 1];
    {
        const StagePoint sp0 = stage_point(g, kmin);
#pragma unroll
        for (int q = 0; q < FB; ++q) pre[q] = stage_load(g, sp0, threadIdx.x + q * blockDim.x);
#pragma unroll
        for (int q = 0; q < FB; ++q) stage_store(g, s_pair[0], s_tm[0], threadIdx.x + q * blockDim.x, pre[q]);
        for (int e = threadIdx.x + FB * blockDim.x; e < TS; e += blockDim.x)
            stage_store(g, s_pair[0], s_tm[0], e, stage_load(g, sp0, e));
    }
    __syncthreads();

    // Work items of a split point: the 8-blocks of the stationary side, `R` of them side by side in a
    // wave (see below).  Whole items go round robin over the waves; the items left over after the last
    // full round are cut into `parts` pieces of their streaming range so that every wave gets one
    // (halves = 0 disables the cutting).
    const int chi = 7; // last column of the block that exists (a block column that is not full lacks its FIRST columns)
    for (int k = kmin; k <= kmax; ++k) {
        const int cur = NBUF == 2 ? (k - kmin) & 1 : 0, nxt = NBUF == 2 ? cur ^ 1 : 0;
        const double2 *pair = s_pair[cur];
        const double *tmv = s_tm[cur];
        const StagePoint spn = stage_point(g, k + 1);
        if (k < kmax) { // records of the next split point: in flight during this pass
#pragma unroll
            for (int q = 0; q < FB; ++q) pre[q] = stage_load(g, spn, threadIdx.x + q * blockDim.x);
        }
        // Lanes of this pass.  Only the rows 0..jr of the block hold states that can be split at k
        // (u + s <= k), and only the columns chi-jc..chi (k <= v - r): near the ends of the block's
        // split range most of the 64 states idle.  Then the wave takes R items at once: the rows (or
        // columns) that matter, padded to a power of two, times R stationary blocks.
        const int jr = k - (ub * 8 + s), jc = vmax - r - k;
        const int nr = imin(jr, 7) + 1, nc = imin(jc, chi) + 1;
        const int lr = nr <= 1 ? 0 : nr <= 2 ? 1 : nr <= 4 ? 2 : 3, lc = nc <= 1 ? 0 : nc <= 2 ? 1 : nc <= 4 ? 2 : 3;
        int R, lgR, slot, ue, ve; // items side by side (and its binary logarithm), this lane's item among them, its row and column
        if (lr <= lc) {      // rows 0..2^lr-1, all columns
            R = 8 >> lr; lgR = 3 - lr; slot = lane >> (3 + lr); ue = (lane >> 3) & ((1 << lr) - 1); ve = lane & 7;
        } else {             // all rows, the last 2^lc columns that exist
            R = 8 >> lc; lgR = 3 - lc; slot = lane >> (3 + lc);
            const int w = lane & ((8 << lc) - 1);
            ue = w >> lc; ve = imax(0, chi - (1 << lc) + 1) + (w & ((1 << lc) - 1));
        }
        // The items of the pass, with (PACK) or without several of them side by side in a wave; the
        // plain variant keeps the item's block, row offset and key column in scalar registers.
        auto run_items = [&](auto pack_c, const int R, const int lgR, const int slot, const int ue, const int ve) {
        constexpr bool PACK = decltype(pack_c)::value;
        const int yl = y_left ? ue : ve, ql = y_left ? ve : ue; // lane index of a streaming / stationary record
        const int col = PACK ? ue * 8 + ve : lane;              // this lane's state: its column of the key table
        // (R is a power of two, a workgroup has at most four waves: no integer division below)
        const int nsup = (nmb + R - 1) >> lgR;
        const int rem = nsup - div_small(nsup, nw) * nw, full = nsup - rem;
        const int parts = ((halves & 3) && rem) ? (rem == 1 ? nw : (nw == 4 && rem == 2) ? 2 : 1) : 1;
        const int nitems = full + rem * parts;
        for (int item = wave; item < nitems; item += nw) {
            const int cut = item >= full, jj = item - full;
            const int jq = div_small(jj, parts);
            const int sb = cut ? full + jq : item, part = cut ? jj - jq * parts : 0, np = cut ? parts : 1;
            // stationary blocks sb R .. sb R + R - 1 (those that exist); this lane's is mb
            const int mb_first = sb * R, mb_last = imin(mb_first + R - 1, nmb - 1);
            // a lane without a block of its own repeats the last block's work for its state: the same
            // candidates into the same keys, which a minimum does not notice (masking them cost 32
            // selects per item)
            const int mb = PACK ? imin(mb_first + slot, mb_last) : sb;
            const int q0 = qM0 + 8 * mb;                // first stationary unit count of this lane's block
            // streaming range: every unit count some block of the item pairs with inside the target
            // group; a lane's surplus steps fall on targets outside the group and are swallowed
            int mlo = imax(yM0, a_g0 - (qM0 + 8 * mb_last + 7)), mhi = imin(yM1, a_g1 - (qM0 + 8 * mb_first));
            if (np > 1 && mlo <= mhi) { // piece `part` of `np` of that range
                const int len = mhi - mlo + 1, lo = mlo + div_small(len * part, np);
                mhi = mlo + div_small(len * (part + 1), np) - 1;
                mlo = lo;
            }
            if (mlo > mhi) continue;
            double bb2[8], bbt[8], btm[8], acc[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int o = fillY + (8 * mb + i) * 8 + ql;
                const double2 p = pair[o];
                bb2[i] = p.x; bbt[i] = p.y; btm[i] = tmv[o];
                acc[i] = kNone;
            }
            const double kd = (double)k;
            const int len = mhi - mlo + 1, j0 = (8 - (len & 7)) & 7;
            int mbase = mlo - j0; // step j of a group handles streaming unit count mbase + j; the first group may start at j0
            const int aoff = q0 - a_g0;
            // one step: the streaming record y against the eight stationary ones, candidates for the
            // targets y + q0 + i, into the rotating minima; then the minimum of target y + q0 is
            // complete for this item.  The streaming record of the NEXT step is read before this
            // step's atomic, so that its latency hides behind the arithmetic (LDS operations
            // complete in order, and the compiler may not move a read over an atomic).
            const double2 *pa = pair + (mlo - yM0) * 8 + yl; // streaming record of the next step
            const double *ta = tmv + (mlo - yM0) * 8 + yl;
            double2 p = *pa;
            double atm = *ta;
#define OOB_STEP(j)                                                                                   \
    {                                                                                                 \
        const int m = mbase + (j);                                                                    \
        pa += 8; ta += 8;                                                                             \
        const double2 pn = *pa; /* may read one record past the last one: staged memory, unused */    \
        const double tn = *ta;                                                                        \
        _Pragma("unroll") for (int i = 0; i < 8; ++i) {                                               \
            const double T = atm >= btm[i] ? p.x + bb2[i] : p.y + bbt[i];                             \
            /* the eighth candidate is the first one of its target: its slot was flushed one step ago */ \
            acc[((j) + i) & 7] = i == 7 ? T : fmin(acc[((j) + i) & 7], T);                            \
        }                                                                                             \
        const int row = imin(imax(m + aoff, -1), na) + 1;                                             \
        atomicMin(&s_acc[row * 64 + col], (unsigned long long)__double_as_longlong(fma(acc[(j)], KS, kd))); \
        p = pn; atm = tn;                                                                             \
    }
            if (j0) {
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if (j >= j0) OOB_STEP(j)
                mbase += 8;
            }
            for (; mbase <= mhi; mbase += 8) {
#pragma unroll
                for (int j = 0; j < 8; ++j) OOB_STEP(j)
            }
#undef OOB_STEP
            // the last step was j = 7 with unit count mhi: minima 0..6 belong to targets mhi + q0 + 1 + i
#pragma unroll
            for (int i = 0; i < 7; ++i) {
                const int row = imin(imax(mhi + 1 + i + aoff, -1), na) + 1;
                atomicMin(&s_acc[row * 64 + col], (unsigned long long)__double_as_longlong(fma(acc[i], KS, kd)));
            }
        }
        };
        if (R > 1 && nmb > 1 && (halves & 4)) run_items(std::true_type{}, R, lgR, slot, ue, ve);
        else run_items(std::false_type{}, 1, 0, 0, lane >> 3, lane & 7);
        if (NBUF == 1) __syncthreads(); // one buffer: everybody is done reading it before it is refilled
        if (k < kmax) {
#pragma unroll
            for (int q = 0; q < FB; ++q)
                stage_store(g, s_pair[nxt], s_tm[nxt], threadIdx.x + q * blockDim.x, pre[q]);
            for (int e = threadIdx.x + FB * blockDim.x; e < TS; e += blockDim.x)
                stage_store(g, s_pair[nxt], s_tm[nxt], e, stage_load(g, spn, e));
        }
        __syncthreads(); // buffer cur fully consumed, buffer cur^1 complete
    }
    // merge into the level's keys: other segments of the same block do the same
    for (int e = threadIdx.x; e < na * 64; e += blockDim.x) {
        const unsigned long long key = s_acc[64 + e];
        if (key == kNoneBits) continue;
        const int aidx = fam_base + a_g0 + (e >> 6) - dlo_of(Sp, M);
        const long long slot = ((long long)(s - 1) * NAall + aidx) * NT + tile;
        atomicMin(&t.partKey[slot * 64 + (e & 63)], key);
    }
}

// Per level: the list of (block, segment) workgroup tasks, written once per call.
// by_row = 0 (default): blocks by decreasing distance from the diagonal, the longest split ranges
// first.  by_row = 1 (handle option OOB_OPT_XCD_ORDER, used together with xcd_chunked): block row ub, then segment,
// then the blocks of that row from the far end, so that neighbours in the list split at the same
// points k and stage the same left-child records.
__device__ void seg_tab_body(const Tables &t, int S, int by_row) {
    if (S > t.sh.Smax || threadIdx.x != 0) return;
    const int L = t.sh.L, NB = nblocks_of(L), ubmax = (L - S) / 8, dmin = tile_dmin(L, S);
    int2 *out = t.seg_tab + (long long)(S - 2) * t.seg_stride;
    int n = 0;
    if (!by_row) {
        int tt = 0;
        for (int d = NB - 1; d >= dmin; --d)
            for (int u = 0; u <= imin(ubmax, NB - 1 - d); ++u, ++tt) {
                const int c = seg_n(tile_krange(L, S, u, u + d), seg_target(L, S));
                for (int j = 0; j < c; ++j) out[n++] = make_int2(tt, u | ((u + d) << 8) | (j << 16));
            }
        return;
    }
    for (int u = 0; u <= imin(ubmax, NB - 1 - dmin); ++u) {
        const int cmax = seg_n(tile_krange(L, S, u, NB - 1), seg_target(L, S)); // the row's longest split range
        for (int j = 0; j < cmax; ++j) {
            int tt = u; // index of block (u, u + d) in tile order: the blocks of all larger d come first
            for (int d = NB - 1; d >= dmin; --d) {
                if (u + d <= NB - 1 && j < seg_n(tile_krange(L, S, u, u + d), seg_target(L, S)))
                    out[n++] = make_int2(tt, u | ((u + d) << 8) | (j << 16));
                tt += imin(ubmax, NB - 1 - d) + 1;
            }
        }
    }
}

// Everything a call needs before level 1, as one launch of kSetupThreads-wide workgroups:
// workgroup 0 the set-up, workgroups 1 .. Smax-1 the task lists of the levels 2 .. Smax, the rest
// set the n keys of the per-split minima to "no such state".  The three parts touch disjoint memory.
__global__ void __launch_bounds__(kSetupThreads) k_prepare(Tables t, oob_profile prof, int force_plain, int by_row,
                                                           unsigned long long *keys, long long n) {
    const int b = blockIdx.x, nseg = imax(t.sh.Smax - 1, 0);
    if (b == 0) { setup_body(t, prof, force_plain); return; }
    if (b <= nseg) { seg_tab_body(t, b + 1, by_row); return; }
    const long long i = (long long)(b - 1 - nseg) * blockDim.x + threadIdx.x;
    if (i < n) keys[i] = 0x7FF0000000000000ull;
}

// ---------------------------------------------------------------------------------------
// Levels S' >= 2, second kernel: grid (block of the plane, delta), one lane per state.
// ---------------------------------------------------------------------------------------
// Loads a lane of k_select keeps in flight: keys of the splits, and pairs of child records while it looks
// for the first m.  With 16 and 4 the kernel needs 98 registers, with 16 and 2 it needs 64 and the call
// is 1 % faster (its waves sit on the chain between the levels and find room beside the split kernels'
// sooner); 8 and 2 the same; one pair or 4 keys at a time: slower again, the kernel's own latency shows.
constexpr int kSelKeys = 16, kSelPairs = 2;
__device__ void select_lane_per_state(const Tables &t, int Sp, int NT, int NAall) {
    const int L = t.sh.L, M = t.sh.M, lane = threadIdx.x;
    int ub, vb;
    tile_decode(L, Sp, blockIdx.x, &ub, &vb);
    const int aidx = blockIdx.y, delta = dlo_of(Sp, M) + aidx;
    const int u = ub * 8 + (lane >> 3), v = vb * 8 + (lane & 7) - t.coff;
    double best = kNone;
    int bs = 0, bk = 0;
    if (t.flags[0]) { // keys total * 2^kbits + k; consumed keys go back to "no such state"
        const double KS = (double)(1 << key_bits(L)), inv = 1.0 / KS;
        const long long o0 = ((long long)aidx * NT + blockIdx.x) * 64 + lane, os = (long long)NAall * NT * 64;
        double bkey = kNone;
        for (int s0 = 1; s0 < Sp; s0 += kSelKeys) { // independent loads in flight
            double key[kSelKeys];
#pragma unroll
            for (int q = 0; q < kSelKeys; ++q) key[q] = s0 + q < Sp ? t.partT[o0 + (s0 + q - 1) * os] : kNone;
#pragma unroll
            for (int q = 0; q < kSelKeys; ++q) {
                const double T = floor(key[q] * inv); // +inf stays +inf
                if (T < best) { best = T; bs = s0 + q; bkey = key[q]; }
            }
        }
        if (best < kNone) bk = (int)(bkey - best * KS);
        for (int s = 1; s < Sp; ++s) t.partT[o0 + (s - 1) * os] = kNone;
    } else if (t.flags[1]) {
        for (int s = 1; s < Sp; ++s) { // first s with the smallest minimum
            const long long o = (((long long)(s - 1) * NAall + aidx) * NT + blockIdx.x) * 64 + lane;
            const double T = t.partT[o];
            if (T < best) { best = T; bs = s; bk = t.partK[o]; }
        }
    }
    Rec out = {kNone, kNone, 0.0, 0.0};
    int ks = 0, ch = 0;
    const Family fam = family_of(delta, M);
    int bm = 0;
    Rec a = out, b = out;
    if (!t.flags[0] && !t.flags[1]) {
        // Totals too large for keys (decided by the set-up kernel from the profile): every candidate
        // (s, k, m) of this state in that order with a strict-minimum update.  Slow, exact, rare.
        if (v <= L && v - u >= Sp)
            for (int s = 1; s < Sp; ++s) {
                const int r = Sp - s;
                int mlo, mhi;
                m_range(fam.fam, fam.units, s, r, M, t.sh.n_max, &mlo, &mhi);
                const double cl = t.sh.Nb > 0 ? -(double)r : 3.0 * r, cr = t.sh.Nb > 0 ? 0.0 : 4.0 * s;
                for (int k = u + s; k <= v - r; ++k)
                    for (int m = mlo; m <= mhi; ++m) {
                        const Rec ra = t.rec[rec_index(t, s, fam.fam_base + m, u, k)];
                        const Rec rb = t.rec[rec_index(t, r, fam.fam_base + fam.units - m, k, v)];
                        const double T = ra.tmax >= rb.tmax ? (ra.T + cl * ra.tmax) + 2.0 * rb.T1
                                                            : ra.T1 + (rb.T + cr * rb.tmax);
                        if (T < best) { best = T; bs = s; bk = k; bm = m; a = ra; b = rb; }
                    }
            }
    } else if (best < kNone) {
        const int r = Sp - bs;
        int mlo, mhi;
        m_range(fam.fam, fam.units, bs, r, M, t.sh.n_max, &mlo, &mhi);
        const double cl = t.sh.Nb > 0 ? -(double)r : 3.0 * r, cr = t.sh.Nb > 0 ? 0.0 : 4.0 * bs;
        // first m whose candidate equals the minimum; kSelPairs candidates' records in flight at a time
        const long long tabA = (t.lvl_tab[bs] - dlo_of(bs, M) + fam.fam_base) * (long long)t.tab_recs +
                               rec_off(u, bk, t.coff, t.NB);
        const long long tabB = (t.lvl_tab[r] - dlo_of(r, M) + fam.fam_base + fam.units) * (long long)t.tab_recs +
                               rec_off(bk, v, t.coff, t.NB);
        for (int m0 = mlo; m0 <= mhi && bm == 0; m0 += kSelPairs) {
            Rec ra[kSelPairs], rb[kSelPairs];
#pragma unroll
            for (int q = 0; q < kSelPairs; ++q) {
                const int m = imin(m0 + q, mhi);
                ra[q] = t.rec[tabA + (long long)m * t.tab_recs];
                rb[q] = t.rec[tabB - (long long)m * t.tab_recs];
            }
#pragma unroll
            for (int q = 0; q < kSelPairs; ++q) {
                const double T = ra[q].tmax >= rb[q].tmax ? (ra[q].T + cl * ra[q].tmax) + 2.0 * rb[q].T1
                                                          : ra[q].T1 + (rb[q].T + cr * rb[q].tmax);
                if (bm == 0 && m0 + q <= mhi && T == best) { bm = m0 + q; a = ra[q]; b = rb[q]; }
            }
        }
    }
    if (best < kNone) {
        if (bm == 0) {
            *t.status = kInternalError;
        } else {
            const int r = Sp - bs;
            const long long oa = rec_index(t, bs, fam.fam_base + bm, u, bk);
            const long long ob = rec_index(t, r, fam.fam_base + fam.units - bm, bk, v);
            out.T = best;
            out.T1 = a.T1 + b.T1;                                                                // Eq. 1
            if (a.tmax >= b.tmax) { out.tmax = a.tmax; ks = t.kstar[oa]; out.T3 = a.T3 + b.T1; } // Eq. 3
            else                  { out.tmax = b.tmax; ks = bs + t.kstar[ob]; out.T3 = b.T3; }
            ch = bs | (bk << 10) | (bm << 21);
        }
    }
    const long long o = rec_block(t, Sp, delta, ub, vb) + lane;
    t.rec[o] = out;
    t.kstar[o] = ks;
    t.choice[o] = ch;
}
__global__ void __launch_bounds__(64) k_select(Tables t, int Sp, int NT, int NAall) {
    select_lane_per_state(t, Sp, NT, NAall);
}

// ---------------------------------------------------------------------------------------
// Levels S' >= 2, second kernel, keyed path: grid (block of the plane, delta, row of the block),
// eight lanes per state (a wave holds the eight states of one row of the block).
//
// The lanes of a state share out what the state has to look at, so that each dependent round trip
// to memory covers eight times as much as it would with one lane per state; the kernel sits on the
// chain between the levels and its duration is made of such round trips.
//   1. FUSE only: the two outer splits s = 1 and s = S'-1, whose one-stage child has a single unit
//      count across nodes (a line of candidates instead of a rectangle), are evaluated here,
//      candidate by candidate from the child records; no split kernel is launched for them.
//   2. The keys of the (other) splits: smallest total, then smallest s (a key holds its smallest k).
//   3. The eight partial minima of a state are merged in the order (T, s, k, m).
//   4. A winner that came from a key does not know its m yet: the lanes test eight m at a time.
//   5. Lane 0 of the state forms the record from the two child records.
// Without keys (flags[0] = 0) the wave of row 0 evaluates the block one lane per state as k_select does.
// ---------------------------------------------------------------------------------------
constexpr int kSel8Keys = 8;   // keys a lane has in flight (64 splits per round of a state)
constexpr int kSel8Outer = 4;  // candidates of the outer splits a lane has in flight
constexpr int kSel8M = 2;      // m a lane tests per round (16 per state)

__device__ __forceinline__ Rec24 load24(const Rec *p) {
    Rec24 r;
    r.a = *(const double2 *)p;
    r.tm = p->tmax;
    return r;
}
// Eq. 1-3 for one candidate from the (T, T1, tmax) of its children.
__device__ __forceinline__ double cand_total(const Rec24 &a, const Rec24 &b, double cl, double cr) {
    return a.tm >= b.tm ? (a.a.x + cl * a.tm) + 2.0 * b.a.y : a.a.y + (b.a.x + cr * b.tm);
}

template <bool FUSE>
__global__ void __launch_bounds__(64) k_select8(Tables t, int Sp, int NT, int NAall) {
    if (t.flags[0] == 0) {
        if (blockIdx.z == 0) select_lane_per_state(t, Sp, NT, NAall);
        return;
    }
    const int L = t.sh.L, M = t.sh.M, lane = threadIdx.x, sub = lane & 7, st = lane >> 3;
    int ub, vb;
    tile_decode(L, Sp, blockIdx.x, &ub, &vb);
    const int aidx = blockIdx.y, delta = dlo_of(Sp, M) + aidx;
    const int tl = blockIdx.z * 8 + st, u = ub * 8 + blockIdx.z, v = vb * 8 + st - t.coff;
    const bool valid = v <= L && v - u >= Sp;
    const Family fam = family_of(delta, M);
    const bool fixed_nb = t.sh.Nb > 0;
    const long long trecs = t.tab_recs;
    double best = kNone;
    unsigned btag = 0xffffffffu; // s << 21 | k << 10 | m (m = 0: not known yet)

    if (FUSE && valid) {
        const int nk = v - u - Sp + 1; // split points u + s .. v - r of either outer split
        for (int side = 0; side < (Sp > 2 ? 2 : 1); ++side) {
            const int s = side ? Sp - 1 : 1, r = Sp - s;
            int mlo, mhi;
            m_range(fam.fam, fam.units, s, r, M, t.sh.n_max, &mlo, &mhi);
            const double cl = fixed_nb ? -(double)r : 3.0 * r, cr = fixed_nb ? 0.0 : 4.0 * s;
            const Rec *baseA = t.rec + (t.lvl_tab[s] - dlo_of(s, M) + fam.fam_base) * trecs;
            const Rec *baseB = t.rec + (t.lvl_tab[r] - dlo_of(r, M) + fam.fam_base + fam.units) * trecs;
            for (int m = mlo; m <= mhi; ++m)
                for (int j0 = sub; j0 < nk; j0 += 8 * kSel8Outer) {
                    Rec24 ra[kSel8Outer], rb[kSel8Outer];
                    int kk[kSel8Outer];
#pragma unroll
                    for (int q = 0; q < kSel8Outer; ++q) { // past the end: the last candidate again
                        const int k = u + s + imin(j0 + 8 * q, nk - 1);
                        kk[q] = k;
                        ra[q] = load24(baseA + m * trecs + rec_off(u, k, t.coff, t.NB));
                        rb[q] = load24(baseB - m * trecs + rec_off(k, v, t.coff, t.NB));
                    }
#pragma unroll
                    for (int q = 0; q < kSel8Outer; ++q) {
                        const double T = cand_total(ra[q], rb[q], cl, cr);
                        const unsigned tag = ((unsigned)s << 21) | ((unsigned)kk[q] << 10) | (unsigned)m;
                        if (T < best || (T == best && tag < btag)) { best = T; btag = tag; }
                    }
                }
        }
    }
    if (valid) { // keys total * 2^kbits + k; consumed keys go back to "no such state"
        const double KS = (double)(1 << key_bits(L)), inv = 1.0 / KS;
        const int s_lo = FUSE ? 2 : 1, s_hi = FUSE ? Sp - 2 : Sp - 1;
        const long long o0 = ((long long)aidx * NT + blockIdx.x) * 64 + tl, os = (long long)NAall * NT * 64;
        for (int s0 = s_lo + sub; s0 <= s_hi; s0 += 8 * kSel8Keys) {
            double key[kSel8Keys];
#pragma unroll
            for (int q = 0; q < kSel8Keys; ++q) {
                const int s = s0 + 8 * q;
                key[q] = s <= s_hi ? t.partT[o0 + (s - 1) * os] : kNone;
            }
#pragma unroll
            for (int q = 0; q < kSel8Keys; ++q) {
                const int s = s0 + 8 * q;
                if (s <= s_hi) t.partT[o0 + (s - 1) * os] = kNone;
            }
#pragma unroll
            for (int q = 0; q < kSel8Keys; ++q) {
                const int s = s0 + 8 * q;
                const double T = floor(key[q] * inv);
                if (T < kNone) {
                    const unsigned tag = ((unsigned)s << 21) | ((unsigned)(int)(key[q] - T * KS) << 10);
                    if (T < best || (T == best && tag < btag)) { best = T; btag = tag; }
                }
            }
        }
    }
    // the eight lanes of a state: smallest (T, s, k, m)
#pragma unroll
    for (int d = 1; d < 8; d <<= 1) {
        const double ob = __shfl_xor(best, d, 64);
        const unsigned ot = (unsigned)__shfl_xor((int)btag, d, 64);
        if (ob < best || (ob == best && ot < btag)) { best = ob; btag = ot; }
    }
    const int bs = (int)(btag >> 21), bk = (int)((btag >> 10) & 2047u);
    int bm = (int)(btag & 1023u);
    if (best < kNone && bm == 0) { // first m whose candidate equals the minimum, eight m side by side
        const int r = Sp - bs;
        int mlo, mhi;
        m_range(fam.fam, fam.units, bs, r, M, t.sh.n_max, &mlo, &mhi);
        const double cl = fixed_nb ? -(double)r : 3.0 * r, cr = fixed_nb ? 0.0 : 4.0 * bs;
        const Rec *baseA = t.rec + (t.lvl_tab[bs] - dlo_of(bs, M) + fam.fam_base) * trecs +
                           rec_off(u, bk, t.coff, t.NB);
        const Rec *baseB = t.rec + (t.lvl_tab[r] - dlo_of(r, M) + fam.fam_base + fam.units) * trecs +
                           rec_off(bk, v, t.coff, t.NB);
        for (int m0 = mlo + sub; m0 - sub <= mhi && bm == 0; m0 += 8 * kSel8M) {
            Rec24 ra[kSel8M], rb[kSel8M];
#pragma unroll
            for (int q = 0; q < kSel8M; ++q) {
                const int m = imin(m0 + 8 * q, mhi);
                ra[q] = load24(baseA + m * trecs);
                rb[q] = load24(baseB - m * trecs);
            }
            int found = 0x7fffffff;
#pragma unroll
            for (int q = kSel8M - 1; q >= 0; --q) {
                const int m = m0 + 8 * q;
                if (m <= mhi && cand_total(ra[q], rb[q], cl, cr) == best) found = m;
            }
#pragma unroll
            for (int d = 1; d < 8; d <<= 1) found = imin(found, __shfl_xor(found, d, 64));
            if (found != 0x7fffffff) bm = found;
        }
    }
    if (sub != 0) return;
    Rec out = {kNone, kNone, 0.0, 0.0};
    int ks = 0, ch = 0;
    if (best < kNone) {
        if (bm == 0) {
            *t.status = kInternalError;
        } else {
            const int r = Sp - bs;
            const long long oa = rec_index(t, bs, fam.fam_base + bm, u, bk);
            const long long ob = rec_index(t, r, fam.fam_base + fam.units - bm, bk, v);
            const Rec a = t.rec[oa], b = t.rec[ob];
            const int ka = t.kstar[oa], kb = t.kstar[ob];
            out.T = best;
            out.T1 = a.T1 + b.T1;                                                     // Eq. 1
            if (a.tmax >= b.tmax) { out.tmax = a.tmax; ks = ka; out.T3 = a.T3 + b.T1; } // Eq. 3
            else                  { out.tmax = b.tmax; ks = bs + kb; out.T3 = b.T3; }
            ch = bs | (bk << 10) | (bm << 21);
        }
    }
    const long long o = rec_block(t, Sp, delta, ub, vb) + tl;
    t.rec[o] = out;
    t.kstar[o] = ks;
    t.choice[o] = ch;
}

// ---------------------------------------------------------------------------------------
// Template extraction ("Choosing the number of stages"): one wave per template size
// n = n_min + blockIdx.x, the lanes share out the stage counts; smallest T, then smallest S.
// ---------------------------------------------------------------------------------------
__global__ void __launch_bounds__(64) k_pick(Tables t, oob_templates out) {
    const int i = blockIdx.x, lane = threadIdx.x;
    const int L = t.sh.L, M = t.sh.M, n = t.sh.n_min + i, delta = M - 2 + n;
    double best = kNone;
    int bestS = 0x7fffffff;
    if (n <= t.sh.n_max)
        for (int S = n + lane; S <= t.sh.Smax; S += 64) { // ascending per lane: the first minimum stays
            if (delta < dlo_of(S, M) || delta > dhi_of(S, M, t.sh.n_max)) continue;
            const double T = t.rec[rec_index(t, S, delta, 0, L)].T;
            if (T < best) { best = T; bestS = S; }
        }
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const double ob = __shfl_xor(best, d, 64);
        const int os = __shfl_xor(bestS, d, 64);
        if (ob < best || (ob == best && os < bestS)) { best = ob; bestS = os; }
    }
    if (lane != 0) return;
    if (!(best < kNone)) bestS = 0;
    out.feasible[i] = bestS > 0;
    out.S[i] = bestS;
    long long T = 0, T1 = 0, T2 = 0, T3 = 0, tm = 0;
    int ks = 0;
    if (bestS > 0) {
        const long long o = rec_index(t, bestS, delta, 0, L);
        const Rec r = t.rec[o];
        T = (long long)best; T1 = (long long)r.T1; T3 = (long long)r.T3; tm = (long long)r.tmax;
        ks = t.kstar[o];
        const long long nb = t.sh.Nb > 0 ? t.sh.Nb : 4LL * bestS;
        T2 = (nb - bestS + ks - 1) * tm; // Eq. 2
    }
    out.T[i] = T; out.T1[i] = T1; out.T2[i] = T2; out.T3[i] = T3; out.tmax[i] = tm; out.kstar[i] = ks;
}

// Stages of each template from the stored (s, k, m) tree: one workgroup per template, one thread
// per stage.  Thread p walks from the root to the p-th leaf (left subtree if p is below the left
// child's stage count, else right with p reduced by it), so the walks of a template run side by
// side and the kernel takes as long as the deepest leaf, not as the whole tree.
// Workgroup `count` only writes the end of the offsets.
__global__ void __launch_bounds__(128) k_backtrack(Tables t, oob_templates out) {
    __shared__ long long s_lvl[OOB_MAX_L + 3];
    __shared__ int s_part[128];
    const int i = blockIdx.x, tid = threadIdx.x, cnt = t.sh.count;
    int part = 0;
    for (int q = tid; q < i && q < cnt; q += blockDim.x) part += out.S[q];
    s_part[tid] = part;
    for (int S = tid; S <= t.sh.Smax + 1; S += blockDim.x) s_lvl[S] = t.lvl_tab[S];
    __syncthreads();
    int off = 0;
    for (int q = 0; q < (int)blockDim.x; ++q) off += s_part[q];
    if (tid == 0) out.stage_off[i] = off;
    if (i >= cnt) return;
    const int S = out.S[i];
    if (S == 0) return;
    const int L = t.sh.L, M = t.sh.M;
    int *begin = out.stage_begin + off + i, *gpus = out.stage_gpus + off;
    for (int p = tid; p < S; p += blockDim.x) {
        int Sq = S, delta = M - 2 + t.sh.n_min + i, u = 0, v = L, pos = p;
        while (Sq > 1) {
            const long long o = (s_lvl[Sq] + (delta - dlo_of(Sq, M))) * t.tab_recs +
                                rec_off(u, v, t.coff, t.NB);
            const int ch = t.choice[o];
            const int s = ch & 1023, k = (ch >> 10) & 2047, m = (ch >> 21) & 1023;
            const Family fam = family_of(delta, M);
            if (s < 1 || s >= Sq) { *t.status = kInternalError; break; }
            if (pos < s) { Sq = s; delta = fam.fam_base + m; v = k; }
            else         { pos -= s; Sq -= s; delta = fam.fam_base + fam.units - m; u = k; }
        }
        begin[p] = u;
        gpus[p] = delta < M - 1 ? delta + 1 : M;
    }
    if (tid == 0) begin[S] = L;
}

// ---------------------------------------------------------------------------------------
// Node specification and coverage (Section 4.1.1, Appendix A), one wave.  The template sizes
// are the consecutive integers n0..n_hi, so c pipelines can use exactly the node counts
// c n0 .. c n_hi; the largest pipeline count whose sizes sum to x is therefore
// c = floor(x / n0) when x <= c n_hi, and x is no sum of sizes at all otherwise (fewer
// pipelines reach even less).  That is the value the coin-change recursion of Section 4.2.1
// gives, without the table.
// ---------------------------------------------------------------------------------------
__global__ void __launch_bounds__(64) k_coverage(Tables t, oob_templates out, int len) {
    __shared__ int s_i0, s_i1, s_thm, s_tail;
    const int cnt = t.sh.count, f = t.sh.f, lane = threadIdx.x;
    if (lane == 0) {
        int i0 = -1;
        for (int q = 0; q < cnt; ++q) if (out.feasible[q]) { i0 = q; break; }
        int i1 = i0;
        while (i0 >= 0 && i1 + 1 < cnt && out.feasible[i1 + 1]) ++i1;
        s_i0 = i0; s_i1 = i1; s_thm = 1; s_tail = 1;
    }
    for (int q = lane; q < len; q += 64) out.cover_maxpipes[q] = 0;
    __syncthreads();
    if (s_i0 < 0) {
        if (lane < 8) out.cover_hdr[lane] = 0;
        return;
    }
    const int n0 = t.sh.n_min + s_i0, n_hi = t.sh.n_min + s_i1, p = n_hi - n0 + 1;
    const int N = n_hi + f * n0;
    const int lo_thm = (f + 1) * n0, lo_tail = N - f < 1 ? 1 : N - f;
    const int lo = lo_thm < lo_tail ? lo_thm : lo_tail;
    for (int x = lo + lane; x <= N; x += 64) {
        int c = x / n0;
        if ((long long)c * n_hi < x) c = 0;
        if (x - lo < len) out.cover_maxpipes[x - lo] = c;
        if (x >= lo_thm && c < f + 1) atomicMin(&s_thm, 0);
        if (x >= lo_tail && c < 1) atomicMin(&s_tail, 0);
    }
    __syncthreads();
    if (lane == 0) {
        out.cover_hdr[0] = n0; out.cover_hdr[1] = n_hi; out.cover_hdr[2] = p; out.cover_hdr[3] = N;
        out.cover_hdr[4] = p > n0 - 1; out.cover_hdr[5] = lo; out.cover_hdr[6] = s_thm; out.cover_hdr[7] = s_tail;
    }
}

// Copies one table into dense n x n arrays, n = L-S'+1, entry [u][v - S'] (tests only).
__global__ void k_export(Tables t, int S, int delta, double *T, double *T1, double *tmax, double *T3,
                         int *kstar, int *choice) {
    const int n = t.sh.L - S + 1;
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= n * n) return;
    const int u = idx / n, j = idx % n, v = j + S;
    Rec r = {kNone, kNone, 0.0, 0.0};
    int ks = 0, ch = 0;
    if (j >= u) {
        const long long o = rec_index(t, S, delta, u, v);
        r = t.rec[o]; ks = t.kstar[o]; ch = t.choice[o];
    }
    T[idx] = r.T; T1[idx] = r.T1; tmax[idx] = r.tmax; T3[idx] = r.T3; kstar[idx] = ks; choice[idx] = ch;
}

// ---------------------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------------------
inline size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

long long table_count(int L, int M, int n_max, int Nb) {
    const int Smax = smax_of(L, n_max, M, Nb);
    long long e = 0;
    for (int S = 1; S <= Smax; ++S) {
        const int nd = dhi_of(S, M, n_max) - dlo_of(S, M) + 1;
        if (nd > 0) e += nd;
    }
    return e;
}

// Largest (S'-1) * deltas * tiles over the levels: slots of the per-split minima.
long long part_slots(int L, int M, int n_max, int Nb) {
    const int Smax = smax_of(L, n_max, M, Nb);
    long long best = 1;
    for (int S = 2; S <= Smax; ++S) {
        const long long nd = dhi_of(S, M, n_max) - dlo_of(S, M) + 1;
        if (nd <= 0) continue;
        const long long sl = (long long)(S - 1) * nd * tile_count_bound(L, S);
        if (sl > best) best = sl;
    }
    return best;
}

struct Carve {
    size_t lvl_tab, PT, PF, PM, rec, kstar, choice, partT, partK, stack, flags, seg_tab, total;
    long long recs, slots;
};
// Byte offsets of the workspace arrays, sized for the handle's maxima.
Carve carve(int L, int nodes, int M) {
    Carve c;
    c.recs = table_count(L, M, nodes, 0) * tri_blocks(nblocks_of(L)) * 64;
    c.slots = part_slots(L, M, nodes, 0);
    const size_t E = (size_t)c.recs;
    const int Smax = smax_of(L, nodes, M, 0);
    size_t o = 0;
    c.lvl_tab = o; o = align_up(o + sizeof(long long) * (OOB_MAX_L + 3));
    c.PT = o;      o = align_up(o + sizeof(long long) * (size_t)(M + 1) * (L + 1));
    c.PF = o;      o = align_up(o + sizeof(int) * (size_t)(M + 1) * (L + 1));
    c.PM = o;      o = align_up(o + sizeof(long long) * (size_t)(L + 1));
    c.rec = o;     o = align_up(o + sizeof(Rec) * E);
    c.kstar = o;   o = align_up(o + sizeof(int) * E);
    c.choice = o;  o = align_up(o + sizeof(int) * E);
    // two buffers of minima: consecutive levels are evaluated side by side (see oob_plan_templates)
    c.partT = o;   o = align_up(o + 2 * sizeof(double) * (size_t)c.slots * 64);
    c.partK = o;   o = align_up(o + sizeof(int) * (size_t)c.slots * 64); // plain kernel only: one stream
    c.stack = o;   o = align_up(o + sizeof(int) * ((size_t)nodes * (Smax + 1) * 4 + nodes + 2));
    c.flags = o;   o = align_up(o + sizeof(int) * 64);
    // the task list of a level is longest at S' = 2; every level gets that many entries
    c.seg_tab = o; o = align_up(o + sizeof(int2) * ((size_t)imax(Smax - 1, 1) * seg_count_bound(L) + 1));
    c.total = o;
    return c;
}

// Structural work counts: states = (u, v) with v - u >= S' per table; candidates = (s, k, m)
// with both children valid: per (s, m) pair one per (u, k, v), u + s <= k <= v - r.
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
                m_range(fam.fam, fam.units, s, S - s, sh.M, sh.n_max, &lo, &hi);
                if (hi >= lo) pairs += hi - lo + 1;
            }
            ca += pairs * (n * (n + 1) * (n + 2) / 6);
        }
    }
    *states = st; *cands = ca;
}

constexpr size_t kLdsLimit = 160 * 1024; // gfx950: 160 KB of LDS per workgroup
constexpr size_t kLdsPrefer = 64 * 1024; // at least two workgroups per compute unit

// Launch shape of k_split for one family of one level.
struct SplitPlan { int waves, groups, pc, cls, ntab, na; size_t lds; };
bool plan_split(const Shape &sh, int Sp, int fam, SplitPlan *p) {
    int t_lo, t_hi;
    target_units(fam, Sp, sh.M, sh.n_max, &t_lo, &t_hi);
    if (fam == 0 && Sp > sh.M) return false;
    if (t_hi < t_lo) return false;
    const int cnt = t_hi - t_lo + 1;
    p->waves = imin(8, cdiv(cnt, 8));
    p->groups = cdiv(cnt, 8 * p->waves);
    int ntab = 1;
    for (int s = 1; s < Sp; ++s) {
        int A_lo, A_hi, B_lo, B_hi;
        child_units(fam, s, sh.M, sh.n_max, &A_lo, &A_hi);
        child_units(fam, Sp - s, sh.M, sh.n_max, &B_lo, &B_hi);
        for (int g = 0; g < p->groups; ++g) {
            const int a0 = t_lo + g * p->waves * 8, a1 = imin(t_hi, a0 + p->waves * 8 - 1);
            const int mA0 = imax(A_lo, a0 - B_hi), mA1 = imin(A_hi, a1 - B_lo);
            const int mB0 = imax(B_lo, a0 - A_hi), mB1 = imin(B_hi, a1 - A_lo);
            if (mA0 <= mA1 && mB0 <= mB1) ntab = imax(ntab, mA1 - mA0 + 1 + mB1 - mB0 + 1 + 1);
        }
    }
    const size_t per_k = (size_t)ntab * 8 * 24;
    p->pc = per_k * 4 <= kLdsPrefer ? 4 : per_k * 2 <= kLdsPrefer ? 2 : 1;
    p->lds = per_k * p->pc;
    return true;
}

// Launch shape of k_split_key for one family of one level.
int env_or(const char *name, int dflt) {
    const char *v = getenv(name);
    return v && *v ? atoi(v) : dflt;
}
// Debug knobs, read once when the library is loaded (the defaults are the measured optimum).
static const int kKeyWaves = env_or("OOB_TUNE_KEY_WAVES", 4);
static const int kKeyHalves = env_or("OOB_TUNE_KEY_HALVES", 2);
static const int kKeyPack = env_or("OOB_TUNE_KEY_PACK", 1);
static const int kBatchOverlap = env_or("OOB_TUNE_BATCH_OVERLAP", 0);
static const int kBatchLanes = env_or("OOB_TUNE_BATCH_LANES", 8);
// From this level on the select kernel works with eight lanes per state and evaluates the two outer
// splits itself (below it the machine is full of split workgroups, and eight times the waves of
// the plain select only wait longer for a place); measured on the headline workload, where 78-88 gave
// the same time.  Handle options move both thresholds.
constexpr int kSelect8From = 82, kFuseFrom = 82;
bool plan_split_key(const Shape &sh, int Sp, int fam, int xcd_order, SplitPlan *p) {
    int t_lo, t_hi;
    target_units(fam, Sp, sh.M, sh.n_max, &t_lo, &t_hi);
    if (fam == 0 && Sp > sh.M) return false;
    if (t_hi < t_lo) return false;
    const int cnt = t_hi - t_lo + 1;
    p->groups = cdiv(cnt, kKeyTargets);
    int ntab = 1;
    for (int s = 1; s < Sp; ++s) {
        int A_lo, A_hi, B_lo, B_hi;
        child_units(fam, s, sh.M, sh.n_max, &A_lo, &A_hi);
        child_units(fam, Sp - s, sh.M, sh.n_max, &B_lo, &B_hi);
        for (int g = 0; g < p->groups; ++g) {
            const int a0 = t_lo + g * kKeyTargets, a1 = imin(t_hi, a0 + kKeyTargets - 1);
            const int mA0 = imax(A_lo, a0 - B_hi), mA1 = imin(A_hi, a1 - B_lo);
            const int mB0 = imax(B_lo, a0 - A_hi), mB1 = imin(B_hi, a1 - A_lo);
            if (mA0 <= mA1 && mB0 <= mB1) { // either child may be the stationary (padded) side
                const int nA = mA1 - mA0 + 1, nB = mB1 - mB0 + 1;
                ntab = imax(ntab, imax(nA + 8 * cdiv(nB, 8), nB + 8 * cdiv(nA, 8)));
            }
        }
    }
    p->pc = (kKeyHalves & 3) | (kKeyPack ? 4 : 0) | (xcd_order ? 8 : 0); // bits 0-1: cut left-over items; bit 2: several items per wave near the range ends; bit 3: XCD-chunked task order
    p->ntab = ntab;
    p->na = imin(cnt, kKeyTargets);
    p->lds = 0; // staged records in static LDS by capacity class, key table in dynamic LDS: see the launch site
    p->waves = kKeyWaves;
    return true;
}

} // namespace oob

using namespace oob;

// The second stream and the events of a handle are borrowed from a pool that lives as long as the
// process and are given back when the handle is destroyed: nothing is created or destroyed per
// handle once the pool is warm (a harness that created and destroyed hundreds of handles, each
// with a stream and events of its own, ended in a host segmentation fault inside the runtime).
struct AuxPool {
    std::mutex mu;
    std::vector<hipStream_t> streams;
    std::vector<hipEvent_t> events;
};
static AuxPool &aux_pool() {
    static AuxPool *p = new AuxPool(); // never destroyed: no order-of-destruction trouble at exit
    return *p;
}
static hipStream_t borrow_stream() {
    AuxPool &p = aux_pool();
    std::lock_guard<std::mutex> lk(p.mu);
    if (!p.streams.empty()) { hipStream_t s = p.streams.back(); p.streams.pop_back(); return s; }
    hipStream_t s = nullptr;
    if (hipStreamCreateWithFlags(&s, hipStreamNonBlocking) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
    return s;
}
static hipEvent_t borrow_event() {
    AuxPool &p = aux_pool();
    std::lock_guard<std::mutex> lk(p.mu);
    if (!p.events.empty()) { hipEvent_t e = p.events.back(); p.events.pop_back(); return e; }
    hipEvent_t e = nullptr;
    if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
    return e;
}

// A lane is one job's worth of workspace plus the streams and events to run a job in it.  Lane 0
// serves oob_plan_templates; oob_plan_templates_batch spreads its jobs over all lanes the caller's
// workspace has room for, so that several (small) jobs fill the GPU side by side.
constexpr int kMaxLanes = 8;
struct Lane {
    hipStream_t main = nullptr;       // lanes >= 1: borrowed; lane 0 runs on the caller's stream
    hipStream_t aux = nullptr;        // streams for the inner splits of the even / odd levels, borrowed
    hipStream_t aux2 = nullptr;       // (null: everything on one stream)
    std::vector<hipEvent_t> ev_level; // [2 S'] "level S' selected", [2 S' + 1] "inner splits of level S' done",
                                      // borrowed
    hipEvent_t ev_join = nullptr;     // lanes >= 1: end of the lane's work in a batch, borrowed
};

struct oob_plan {
    int max_L, max_nodes, max_M;
    char *ws;
    size_t ws_bytes;
    Carve cv;
    int lanes;        // workspace_bytes / bytes of one job, at most kMaxLanes
    size_t lane_bytes;
    Lane lane[kMaxLanes];
    hipEvent_t ev_fork; // start of a batch, borrowed at the first batch
    Shape last;       // shape of the last call (for oob_plan_export_block)
    int last_lane;    // and the lane it ran in
    bool have_last;
    hipEvent_t ev_begin, ev_end; // optional: recorded around the level launches
    bool timed;
    int opt_plain, opt_xcd, opt_one_stream, opt_select8_from, opt_fuse_from; // oob_plan_set_option
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
    p->lane_bytes = align_up(cv.total);
    p->lanes = (int)std::min<size_t>(kMaxLanes, std::max<size_t>(1, workspace_bytes / p->lane_bytes));
    p->ev_fork = nullptr; p->last_lane = 0;
    p->opt_plain = p->opt_xcd = p->opt_one_stream = 0;
    p->opt_select8_from = kSelect8From; p->opt_fuse_from = kFuseFrom;
    *h = p;
    return OOB_OK;
}

extern "C" int oob_plan_destroy(oob_plan *h) {
    if (!h) return OOB_EINVAL;
    if (h->ev_begin) { (void)hipEventDestroy(h->ev_begin); (void)hipEventDestroy(h->ev_end); }
    { // the caller has waited for the handle's work: its stream and events go back to the pool
        AuxPool &p = aux_pool();
        std::lock_guard<std::mutex> lk(p.mu);
        for (Lane &ln : h->lane) {
            for (hipEvent_t e : ln.ev_level) p.events.push_back(e);
            if (ln.ev_join) p.events.push_back(ln.ev_join);
            if (ln.aux) p.streams.push_back(ln.aux);
            if (ln.aux2) p.streams.push_back(ln.aux2);
            if (ln.main) p.streams.push_back(ln.main);
        }
        if (h->ev_fork) p.events.push_back(h->ev_fork);
    }
    delete h;
    return OOB_OK;
}

static Tables make_tables(const oob_plan *h, int lane, const Shape &sh, int *status) {
    Tables t;
    char *ws = h->ws + (size_t)lane * h->lane_bytes;
    t.sh = sh;
    t.NB = nblocks_of(sh.L);
    t.coff = col_shift(sh.L);
    t.tab_recs = tri_blocks(t.NB) * 64;
    t.lvl_tab = (long long *)(ws + h->cv.lvl_tab);
    t.PT = (long long *)(ws + h->cv.PT);
    t.PF = (int *)(ws + h->cv.PF);
    t.PM = (long long *)(ws + h->cv.PM);
    t.rec = (Rec *)(ws + h->cv.rec);
    t.kstar = (int *)(ws + h->cv.kstar);
    t.choice = (int *)(ws + h->cv.choice);
    t.partT = (double *)(ws + h->cv.partT);
    t.partKey = (unsigned long long *)(ws + h->cv.partT);
    t.partK = (int *)(ws + h->cv.partK);
    t.stack = (int *)(ws + h->cv.stack);
    t.flags = (int *)(ws + h->cv.flags);
    t.seg_tab = (int2 *)(ws + h->cv.seg_tab);
    t.seg_stride = seg_count_bound(sh.L);
    t.status = status;
    return t;
}

static bool out_ok(const oob_templates *o) {
    return o && o->feasible && o->S && o->kstar && o->T && o->T1 && o->T2 && o->T3 && o->tmax &&
           o->stage_off && o->stage_begin && o->stage_gpus && o->cover_hdr && o->cover_maxpipes &&
           o->status;
}

// The splits s0, s0 + sstep, ... (scount of them) of level S.
struct SplitRange { int s0, sstep, scount; };
// Waves per workgroup of a keyed launch: as many as the split with the most work items (8-blocks of
// the stationary side) offers per split point, at most kKeyWaves.  The low levels have one or two
// items per split point: more waves would only idle at the barriers and take up residency.
static int waves_for(const Shape &sh, int S, int fam, const SplitPlan &sp, SplitRange sr) {
    int t_lo, t_hi;
    target_units(fam, S, sh.M, sh.n_max, &t_lo, &t_hi);
    int most = 1;
    for (int i = 0; i < sr.scount; ++i) {
        const int s = sr.s0 + i * sr.sstep, r = S - s;
        int A_lo, A_hi, B_lo, B_hi;
        child_units(fam, s, sh.M, sh.n_max, &A_lo, &A_hi);
        child_units(fam, r, sh.M, sh.n_max, &B_lo, &B_hi);
        for (int g = 0; g < sp.groups; ++g) {
            const int a0 = t_lo + g * kKeyTargets, a1 = imin(t_hi, a0 + kKeyTargets - 1);
            const int mA0 = imax(A_lo, a0 - B_hi), mA1 = imin(A_hi, a1 - B_lo);
            const int mB0 = imax(B_lo, a0 - A_hi), mB1 = imin(B_hi, a1 - A_lo);
            if (mA0 > mA1 || mB0 > mB1) continue;
            const bool y_left = role_cost(mA0, mA1, mB0, mB1, a0, a1) <= role_cost(mB0, mB1, mA0, mA1, a0, a1);
            most = imax(most, cdiv(y_left ? mB1 - mB0 + 1 : mA1 - mA0 + 1, 8));
        }
    }
    return imin(kKeyWaves, most);
}

// LDS of a keyed launch: the staged records of one split point (static, by capacity class NTAB of the
// tables staged) and the key table of the launch's own target count (dynamic).  A launch whose
// workgroups fit a compute unit's LDS four times runs the variant held to 128 registers (four
// waves per SIMD), else the one with three records in flight (three waves per SIMD either way).
static const int kKeyClasses[] = {24, 32, 48, 64, 96, 136};
static int key_class(int ntab, int na) {
    (void)na;
    for (int c = 0; c < 6; ++c)
        if (ntab <= kKeyClasses[c]) return c;
    return -1;
}
static size_t key_table_bytes(int na) { return (size_t)(na + 2) * 64 * sizeof(unsigned long long); }
// A keyed launch: the target groups of family `fam` (gz of them) and, in a launch for both families
// of a low level, those of the whole-node family behind them (`groups` in all).
struct KeyLaunch { int fam, gz, groups, cls, na, pc, waves; };
template <int NTAB>
static void launch_split_key_c(const Tables &t, int S, const KeyLaunch &kl, int NT, int NAall, SplitRange sr,
                               hipStream_t st) {
    const dim3 grid(seg_count(t.sh.L, S), sr.scount, kl.groups);
    const size_t dyn = key_table_bytes(kl.na), total = (size_t)NTAB * 8 * 24 + dyn;
    if (4 * total <= kLdsLimit)
        hipLaunchKernelGGL((k_split_key<NTAB, 1, kFillBatchSmall>), grid, dim3(kl.waves * 64), dyn, st, t, S, kl.fam, kl.gz, NT, NAall,
                           kl.pc, sr.s0, sr.sstep);
    else
        hipLaunchKernelGGL((k_split_key<NTAB, 1, kFillBatch>), grid, dim3(kl.waves * 64), dyn, st, t, S, kl.fam, kl.gz, NT,
                           NAall, kl.pc, sr.s0, sr.sstep);
}
static void launch_split_key(const Tables &t, int S, const KeyLaunch &kl, int NT, int NAall, SplitRange sr,
                             hipStream_t st) {
    if (sr.scount < 1) return;
    switch (kl.cls) {
    case 0: launch_split_key_c<24>(t, S, kl, NT, NAall, sr, st); break;
    case 1: launch_split_key_c<32>(t, S, kl, NT, NAall, sr, st); break;
    case 2: launch_split_key_c<48>(t, S, kl, NT, NAall, sr, st); break;
    case 3: launch_split_key_c<64>(t, S, kl, NT, NAall, sr, st); break;
    case 4: launch_split_key_c<96>(t, S, kl, NT, NAall, sr, st); break;
    default: launch_split_key_c<136>(t, S, kl, NT, NAall, sr, st); break;
    }
}
// The keyed launches of the splits `sr` of a level: one per family, or one for both.
static void launch_split_keys(const Tables &t, int S, const bool *have, const SplitPlan *kp, int NT, int NAall,
                              SplitRange sr, hipStream_t st) {
    if (sr.scount < 1) return;
    KeyLaunch kl[2];
    for (int fam = 0; fam < 2; ++fam)
        if (have[fam])
            kl[fam] = KeyLaunch{fam, kp[fam].groups, kp[fam].groups, kp[fam].cls, kp[fam].na, kp[fam].pc,
                                waves_for(t.sh, S, fam, kp[fam], sr)};
    if (have[0] && have[1]) {
        const KeyLaunch both{0, kl[0].groups, kl[0].groups + kl[1].groups, imax(kl[0].cls, kl[1].cls),
                             imax(kl[0].na, kl[1].na), kl[0].pc, imax(kl[0].waves, kl[1].waves)};
        launch_split_key(t, S, both, NT, NAall, sr, st);
        return;
    }
    for (int fam = 0; fam < 2; ++fam)
        if (have[fam]) launch_split_key(t, S, kl[fam], NT, NAall, sr, st);
}

template <int PC>
static void launch_split(const Tables &t, int S, int fam, const SplitPlan &sp, int NT, int NAall,
                         hipStream_t st) {
    if (sp.lds > kLdsPrefer) // beyond the default dynamic-LDS limit of a launch
        (void)hipFuncSetAttribute((const void *)k_split<PC>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                  (int)kLdsLimit);
    hipLaunchKernelGGL(k_split<PC>, dim3(NT, S - 1, sp.groups), dim3(sp.waves * 64), sp.lds, st, t, S, fam,
                       NT, NAall);
}

// One job in lane `ln` of the handle, enqueued on `st` (and on the lane's second stream when the
// levels overlap).
static int enqueue_job(oob_plan *h, int ln, bool want_overlap, const oob_profile *profile, int L, int n_min,
                       int n_max, int gpus_per_node, int microbatches, int64_t mem_cap, int f,
                       oob_templates *out, hipStream_t st) {
    if (!h || !profile || !out_ok(out)) return OOB_EINVAL;
    Lane &lane = h->lane[ln];
    if (!profile->fwd_ns || !profile->bwd_ns || !profile->mem_bytes || !profile->boundary_ns) return OOB_EINVAL;
    if (L < 1 || n_min < 1 || n_min > n_max || gpus_per_node < 1 || microbatches < 0 || f < 0 || mem_cap <= 0)
        return OOB_EINVAL;
    if (L > h->max_L || n_max > h->max_nodes || gpus_per_node > h->max_M) return OOB_ECAPACITY;
    if ((long long)n_max * ((long long)f + 1) > (1 << 24)) return OOB_ECAPACITY;
    const int M = gpus_per_node;
    if (table_count(L, M, n_max, microbatches) * tri_blocks(nblocks_of(L)) * 64 > h->cv.recs ||
        part_slots(L, M, n_max, microbatches) > h->cv.slots)
        return OOB_ECAPACITY;
    Shape sh;
    sh.L = L; sh.M = M; sh.n_min = n_min; sh.n_max = n_max; sh.Nb = microbatches; sh.f = f;
    sh.cap = mem_cap; sh.count = n_max - n_min + 1;
    sh.Smax = smax_of(L, n_max, M, microbatches);
    // launch shapes first, so that nothing is enqueued when a level cannot be staged in LDS
    // a level's tables exceed the keyed kernel's LDS classes (or the debug knob says so): plain kernel everywhere
    int force_plain = h->opt_plain != 0;
    for (int S = 2; S <= sh.Smax; ++S)
        for (int fam = 0; fam < 2; ++fam) {
            SplitPlan sp;
            if (plan_split_key(sh, S, fam, h->opt_xcd, &sp) && key_class(sp.ntab, sp.na) < 0) force_plain = 1;
        }
    if (force_plain)
        for (int S = 2; S <= sh.Smax; ++S)
            for (int fam = 0; fam < 2; ++fam) {
                SplitPlan sp;
                if (plan_split(sh, S, fam, &sp) && sp.lds > kLdsLimit) return OOB_ECAPACITY;
            }
    const Tables t = make_tables(h, ln, sh, (int *)out->status);
    work_counts(sh, (long long *)&out->states, (long long *)&out->candidates);

    const long long slot_stride = h->cv.slots * 64; // distance between the two buffers of per-split minima
    hipLaunchKernelGGL(k_prepare, dim3((unsigned)(1 + imax(sh.Smax - 1, 0) + (2 * slot_stride + kSetupThreads - 1) / kSetupThreads)),
                       dim3(kSetupThreads), 0, st, t, *profile, force_plain, h->opt_xcd, t.partKey, 2 * slot_stride);
    hipLaunchKernelGGL(k_level1, dim3(tile_count(L, 1), M), dim3(64), 0, st, t,
                       (const long long *)profile->boundary_ns);
    // Levels.  Level S' depends on the lower levels like this: its inner splits 2 <= s <= S'-2 read the
    // levels up to S'-2 only, its two outer splits (s = 1 and S'-1) read level S'-1, and its select
    // needs all its splits.  So the chain that cannot be shortened is outer splits -> select ->
    // outer splits of the next level ..., two small launches per level, and it runs on the caller's
    // stream.  The inner splits, nearly all of the arithmetic, run on two streams of the library (even
    // and odd levels), each launch waiting for the select of level S'-2 and awaited by the select of its
    // own level; they fill the machine around the chain.  Each parity has its own buffer of per-split
    // minima (a select hands its buffer back reset before the inner splits of level S'+2 start).
    bool overlap = want_overlap && !force_plain && sh.Smax >= 4;
    if (overlap && !lane.aux) lane.aux = borrow_stream();
    if (overlap && !lane.aux2) lane.aux2 = borrow_stream();
    if (overlap && lane.aux && lane.aux2) {
        while ((int)lane.ev_level.size() < 2 * sh.Smax + 2) {
            hipEvent_t e = borrow_event();
            if (!e) break;
            lane.ev_level.push_back(e);
        }
    }
    overlap = overlap && lane.aux && lane.aux2 && (int)lane.ev_level.size() >= 2 * sh.Smax + 2;
    const bool timed = ln == 0 && h->ev_begin;
    if (timed) OOB_HIP_CHECK(hipEventRecord(h->ev_begin, st));
    for (int S = 2; S <= sh.Smax; ++S) {
        const int NAall = dhi_of(S, M, n_max) - dlo_of(S, M) + 1;
        if (NAall <= 0) continue;
        const int NT = tile_count(L, S);
        Tables tl = t; // this level's buffer of per-split minima
        tl.partT = t.partT + (S & 1) * slot_stride;
        tl.partKey = t.partKey + (S & 1) * slot_stride;
        SplitPlan sp[2], kp[2];
        bool have[2];
        for (int fam = 0; fam < 2; ++fam) {
            have[fam] = plan_split(sh, S, fam, &sp[fam]) && plan_split_key(sh, S, fam, h->opt_xcd, &kp[fam]);
            if (have[fam]) kp[fam].cls = key_class(kp[fam].ntab, kp[fam].na);
        }
        const bool inner = overlap && S >= 4;
        if (inner) {
            hipStream_t sx = (S & 1) ? lane.aux2 : lane.aux;
            OOB_HIP_CHECK(hipStreamWaitEvent(sx, lane.ev_level[2 * (S - 2)], 0)); // select of level S'-2
            launch_split_keys(tl, S, have, kp, NT, NAall, SplitRange{2, 1, S - 3}, sx);
            OOB_HIP_CHECK(hipEventRecord(lane.ev_level[2 * S + 1], sx));
        }
        // the outer splits: launches of their own, or evaluated by the select kernel itself
        const bool fuse = !force_plain && S >= h->opt_fuse_from;
        if (!force_plain) {
            SplitRange sr = inner ? SplitRange{1, S - 2, 2} : SplitRange{1, 1, S - 1};
            if (fuse) sr = inner ? SplitRange{1, 1, 0} : SplitRange{2, 1, S - 3};
            launch_split_keys(tl, S, have, kp, NT, NAall, sr, st);
        }
        for (int fam = 0; fam < 2 && force_plain; ++fam) {
            if (!have[fam]) continue;
            if (sp[fam].pc == 4) launch_split<4>(tl, S, fam, sp[fam], NT, NAall, st);
            else if (sp[fam].pc == 2) launch_split<2>(tl, S, fam, sp[fam], NT, NAall, st);
            else launch_split<1>(tl, S, fam, sp[fam], NT, NAall, st);
        }
        if (inner) OOB_HIP_CHECK(hipStreamWaitEvent(st, lane.ev_level[2 * S + 1], 0));
        if (force_plain || (!fuse && S < h->opt_select8_from)) hipLaunchKernelGGL(k_select, dim3(NT, NAall), dim3(64), 0, st, tl, S, NT, NAall);
        else if (fuse) hipLaunchKernelGGL(k_select8<true>, dim3(NT, NAall, 8), dim3(64), 0, st, tl, S, NT, NAall);
        else hipLaunchKernelGGL(k_select8<false>, dim3(NT, NAall, 8), dim3(64), 0, st, tl, S, NT, NAall);
        if (overlap) OOB_HIP_CHECK(hipEventRecord(lane.ev_level[2 * S], st));
    }
    if (timed) { OOB_HIP_CHECK(hipEventRecord(h->ev_end, st)); h->timed = true; }
    hipLaunchKernelGGL(k_pick, dim3(sh.count), dim3(64), 0, st, t, *out);
    hipLaunchKernelGGL(k_backtrack, dim3(sh.count + 1), dim3(128), 0, st, t, *out);
    const int len = sh.count > f + 1 ? sh.count : f + 1;
    hipLaunchKernelGGL(k_coverage, dim3(1), dim3(64), 0, st, t, *out, len);
    OOB_HIP_CHECK(hipGetLastError());
    h->last = sh;
    h->last_lane = ln;
    h->have_last = true;
    return OOB_OK;
}

extern "C" int oob_plan_templates(oob_plan *h, const oob_profile *profile, int L, int n_min, int n_max,
                                  int gpus_per_node, int microbatches, int64_t mem_cap, int f,
                                  oob_templates *out, void *stream) {
    return enqueue_job(h, 0, h && !h->opt_one_stream, profile, L, n_min, n_max, gpus_per_node, microbatches, mem_cap, f,
                       out, (hipStream_t)stream);
}

extern "C" int oob_plan_templates_batch(oob_plan *h, int count, const oob_profile *profiles, const int *L,
                                        const int *n_min, const int *n_max, const int *gpus_per_node,
                                        const int *microbatches, const int64_t *mem_cap, const int *f,
                                        oob_templates *outs, void *stream) {
    if (!h || count < 0 || (count > 0 && (!profiles || !L || !n_min || !n_max || !gpus_per_node ||
                                           !microbatches || !mem_cap || !f || !outs)))
        return OOB_EINVAL;
    const int want_overlap = !h->opt_one_stream, lane_overlap = kBatchOverlap, max_lanes = kBatchLanes;
    hipStream_t st = (hipStream_t)stream;
    // Lanes: job i runs in lane i mod K, the jobs of a lane one after the other on the lane's own
    // stream, the lanes side by side.  Lane 0 is the caller's stream; the others start after what
    // the caller has enqueued so far (fork event) and the caller's stream waits for them at the end.
    int K = std::max(1, std::min(std::min(h->lanes, max_lanes), count));
    if (K > 1 && !h->ev_fork) h->ev_fork = borrow_event();
    if (K > 1 && !h->ev_fork) K = 1;
    for (int ln = 1; ln < K; ++ln) {
        Lane &lane = h->lane[ln];
        if (!lane.main) lane.main = borrow_stream();
        if (!lane.ev_join) lane.ev_join = borrow_event();
        if (!lane.main || !lane.ev_join) { K = ln; break; }
    }
    if (K > 1) {
        OOB_HIP_CHECK(hipEventRecord(h->ev_fork, st));
        for (int ln = 1; ln < K; ++ln) OOB_HIP_CHECK(hipStreamWaitEvent(h->lane[ln].main, h->ev_fork, 0));
    }
    int rc = OOB_OK;
    for (int i = 0; i < count && rc == OOB_OK; ++i) {
        const int ln = i % K;
        rc = enqueue_job(h, ln, K > 1 ? lane_overlap != 0 : want_overlap != 0, &profiles[i], L[i], n_min[i], n_max[i],
                         gpus_per_node[i], microbatches[i], mem_cap[i], f[i], &outs[i], ln ? h->lane[ln].main : st);
    }
    for (int ln = 1; ln < K; ++ln) { // also after an error: the caller's stream covers all that was enqueued
        OOB_HIP_CHECK(hipEventRecord(h->lane[ln].ev_join, h->lane[ln].main));
        OOB_HIP_CHECK(hipStreamWaitEvent(st, h->lane[ln].ev_join, 0));
    }
    return rc;
}

extern "C" int oob_plan_set_option(oob_plan *h, int option, int value) {
    if (!h) return OOB_EINVAL;
    switch (option) {
    case OOB_OPT_PLAIN_SPLIT: h->opt_plain = value != 0; break;
    case OOB_OPT_XCD_ORDER: h->opt_xcd = value != 0; break;
    case OOB_OPT_ONE_STREAM: h->opt_one_stream = value != 0; break;
    case OOB_OPT_SELECT8_FROM: h->opt_select8_from = value; break;
    case OOB_OPT_FUSE_FROM: h->opt_fuse_from = value; break;
    default: return OOB_EINVAL;
    }
    return OOB_OK;
}

extern "C" int oob_plan_level_timing(oob_plan *h, int enable) {
    if (!h) return OOB_EINVAL;
    if (enable && !h->ev_begin) {
        OOB_HIP_CHECK(hipEventCreate(&h->ev_begin));
        OOB_HIP_CHECK(hipEventCreate(&h->ev_end));
    } else if (!enable && h->ev_begin) {
        (void)hipEventDestroy(h->ev_begin); (void)hipEventDestroy(h->ev_end);
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

// Measurement: sixteen independent chains of 32-bit add / compare / select per lane, the
// operation mix the roofline of the level kernels is quoted in.  3 lane-operations per chain step.
__global__ void __launch_bounds__(256) k_valu_peak(int *sink, int iters, int a, int b) {
    int v[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) v[i] = threadIdx.x + i * a;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int w = v[i] + a;
            v[i] = w > b ? w : v[i];
        }
    }
    int r = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) r ^= v[i];
    if (r == 0x7fffffff) sink[0] = r; // keeps the chains alive; practically never taken
}

// Measurement: the instruction mix of a candidate of the split kernels in fp64, eight candidates per
// step as there (two adds, a compare, a 64-bit select, a min against a running minimum each), plus
// the three adds that change the step's streaming values.  51 lane-instructions per step.
__global__ void __launch_bounds__(256) k_valu_peak_f64(double *sink, int iters, double a, double b) {
    double bb2[8], bbt[8], btm[8], acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        bb2[i] = a * (threadIdx.x + i); bbt[i] = b * (threadIdx.x + 2 * i); btm[i] = a * b * (3 * i + (threadIdx.x & 7));
        acc[i] = 1e300;
    }
    double px = a, py = b, atm = a + b;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const double T = atm >= btm[i] ? px + bb2[i] : py + bbt[i];
            acc[i] = fmin(acc[i], T);
        }
        px += a; py += b; atm += a;
    }
    double r = 0.0;
#pragma unroll
    for (int i = 0; i < 8; ++i) r += acc[i];
    if (r == 12345.678) sink[0] = r; // keeps the chains alive; practically never taken
}

// Host-side check of the table layout and the task lists for L layers (no GPU involved): every state
// (S', u, v) lies in exactly one enumerated block of its level and at a record of its own, every
// enumerated block holds a state, the segments of a block partition its split range into parts of at
// least one split point, and the counts stay within the bounds that size a workspace.
extern "C" int oob_plan_layout_selftest(int L) {
    if (L < 1 || L > OOB_MAX_L) return OOB_EINVAL;
    const int NB = nblocks_of(L), c = col_shift(L), recs = tri_blocks(NB) * 64;
    if ((L + c + 1) % 8 != 0 || (L + c) / 8 != NB - 1) return 1;
    std::vector<int> owner((size_t)(L + 1) * (L + 1));
    std::vector<char> used(recs);
    for (int u = 0; u <= L; ++u) // records of distinct (u, v) are distinct and inside the table
        for (int v = u; v <= L; ++v) {
            const int o = rec_off(u, v, c, NB);
            if (o < 0 || o >= recs || used[o]) return 2;
            used[o] = 1;
        }
    for (int S = 1; S <= L; ++S) {
        std::fill(owner.begin(), owner.end(), -1);
        const int nt = tile_count(L, S);
        if (nt > tile_count_bound(L, S)) return 3;
        int segs = 0;
        for (int t = 0; t < nt; ++t) {
            int ub, vb;
            tile_decode(L, S, t, &ub, &vb);
            if (ub < 0 || vb < ub || vb >= NB) return 4;
            const int kr = tile_krange(L, S, ub, vb);
            if (kr < 1 || tile_vmax(L, vb) > L) return 5;
            const int n = seg_n(kr, seg_target(L, S));
            int next = 0;
            for (int j = 0; j < n; ++j) {
                int ofs, len;
                seg_span(kr, n, j, &ofs, &len);
                if (ofs != next || len < 1) return 6;
                next = ofs + len;
            }
            if (next != kr) return 6;
            segs += n;
            int states = 0;
            for (int u = ub * 8; u < ub * 8 + 8; ++u)
                for (int v = vb * 8 - c; v <= vb * 8 + 7 - c; ++v) {
                    if (u >= L || v < 0 || v > L || v - u < S) continue;
                    if (owner[(size_t)u * (L + 1) + v] != -1) return 7;
                    owner[(size_t)u * (L + 1) + v] = t;
                    if (rec_off(u, v, c, NB) != tri_index(ub, vb, NB) * 64 + ((u - ub * 8) << 3) + (v + c - vb * 8)) return 8;
                    ++states;
                }
            if (states == 0) return 9;
        }
        for (int u = 0; u < L; ++u)
            for (int v = u + S; v <= L; ++v)
                if (owner[(size_t)u * (L + 1) + v] < 0) return 10;
        if (S >= 2 && (segs != seg_count(L, S) || segs > seg_count_bound(L))) return 11;
    }
    return 0;
}

// Copies flags[0..3] of the last call to a device array (tests: which split kernel ran).
__global__ void k_export_flags(const int *flags, int *dst) {
    if (threadIdx.x < 4) dst[threadIdx.x] = flags[threadIdx.x];
}

extern "C" int oob_plan_export_flags(oob_plan *h, int32_t *flags, void *stream) {
    if (!h || !h->have_last || !flags) return OOB_EINVAL;
    hipLaunchKernelGGL(k_export_flags, dim3(1), dim3(64), 0, (hipStream_t)stream, (const int *)(h->ws + (size_t)h->last_lane * h->lane_bytes + h->cv.flags),
                       (int *)flags);
    OOB_HIP_CHECK(hipGetLastError());
    return OOB_OK;
}

extern "C" int oob_plan_export_block(oob_plan *h, int S, int delta, double *T, double *T1, double *tmax,
                                     double *T3, int32_t *kstar, int32_t *choice, void *stream) {
    if (!h || !h->have_last || !T || !T1 || !tmax || !T3 || !kstar || !choice) return OOB_EINVAL;
    const Shape &sh = h->last;
    if (S < 1 || S > sh.Smax) return OOB_EINVAL;
    if (delta < dlo_of(S, sh.M) || delta > dhi_of(S, sh.M, sh.n_max)) return OOB_EINVAL;
    const Tables t = make_tables(h, h->last_lane, sh, nullptr);
    const int n = sh.L - S + 1;
    hipLaunchKernelGGL(k_export, dim3((n * n + 255) / 256), dim3(256), 0, (hipStream_t)stream, t, S, delta, T,
                       T1, tmax, T3, (int *)kstar, (int *)choice);
    OOB_HIP_CHECK(hipGetLastError());
    return OOB_OK;
}

// Measured vector-ALU peak of this GPU in lane-operations per second, for comparison with the nominal
// 256 CUs x 64 lanes x clock: 32-bit add / compare / select (f64_mix = 0) or the fp64 instruction mix
// of a candidate of the split kernels (f64_mix = 1).
static int valu_peak(oob_plan *h, void *stream, double *lane_ops_per_s, int f64_mix) {
    if (!h || !lane_ops_per_s) return OOB_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    hipEvent_t e0, e1;
    OOB_HIP_CHECK(hipEventCreate(&e0));
    OOB_HIP_CHECK(hipEventCreate(&e1));
    const int iters = f64_mix ? 6000 : 20000, grid = 256 * 32; // 32 workgroups of 4 waves per compute unit
    int *sink = (int *)(h->ws + h->cv.flags) + 32; // spare words of the flags array (8-byte aligned)
    for (int pass = 0; pass < 2; ++pass) { // warm-up, then the timed launch
        if (pass) OOB_HIP_CHECK(hipEventRecord(e0, st));
        if (f64_mix) hipLaunchKernelGGL(k_valu_peak_f64, dim3(grid), dim3(256), 0, st, (double *)sink, pass ? iters : 100, 1.0, 3.0);
        else         hipLaunchKernelGGL(k_valu_peak, dim3(grid), dim3(256), 0, st, sink, pass ? iters : 100, 1, 1 << 30);
    }
    OOB_HIP_CHECK(hipEventRecord(e1, st));
    OOB_HIP_CHECK(hipEventSynchronize(e1));
    float ms = 0.f;
    OOB_HIP_CHECK(hipEventElapsedTime(&ms, e0, e1));
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    *lane_ops_per_s = (double)grid * 256 * (f64_mix ? 51.0 : 16.0 * 3) * iters / (ms * 1e-3);
    return OOB_OK;
}
extern "C" int oob_plan_valu_peak(oob_plan *h, void *stream, double *lane_ops_per_s) {
    return valu_peak(h, stream, lane_ops_per_s, 0);
}
extern "C" int oob_plan_valu_peak_f64(oob_plan *h, void *stream, double *lane_ops_per_s) {
    return valu_peak(h, stream, lane_ops_per_s, 1);
}
