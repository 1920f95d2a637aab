// Table layout and index arithmetic shared by the host driver and the kernels.
//
// Notation (Section 4.1.2 of the paper): a state is (S', u, v, delta): layers [u, v) cut into
// S' stages on device set delta.  Device sets: G(g) = g GPUs inside one node (delta = g-1,
// 1 <= g <= M-1) and A(a) = a whole nodes (delta = M-2+a).  Both kinds form an additive
// family: a set of `units` is split into m and units-m, with delta = fam_base + units where
// fam_base = -1 inside a node (units = GPUs, A(1) counts as M GPUs) and M-2 across nodes
// (units = nodes).
//
// Level S' stores, for every delta in [dlo(S'), dhi(S')], a dense n x n block, n = L-S'+1,
// record (u, v) at row i = u, column j = v - S'; only j >= i are states, the rest is padding
// that holds the "no such state" value so that the inner loops need no masks.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace oob {

struct Shape {
    int L, M, n_min, n_max, Nb, f, Smax, count;
    long long cap;
};

__host__ __device__ inline int imin(int a, int b) { return a < b ? a : b; }
__host__ __device__ inline int imax(int a, int b) { return a > b ? a : b; }

// (S', delta) exists ("Choosing the number of stages": a stage never spans nodes and every
// GPU is used): G(g): S' <= g;  A(a): a <= S' <= a*M.  The valid deltas of a level are the
// contiguous range [dlo, dhi].
__host__ __device__ inline int dlo_of(int S, int M) {
    return S <= M ? S - 1 : M - 2 + (S + M - 1) / M;
}
__host__ __device__ inline int dhi_of(int S, int M, int n_max) { return M - 2 + imin(S, n_max); }

__host__ __device__ inline int smax_of(int L, int n_max, int M, int Nb) {
    long long s = L;
    if ((long long)n_max * M < s) s = (long long)n_max * M;
    if (Nb > 0 && Nb < s) s = Nb;
    return (int)s;
}

// Family of a target device set.
struct Family {
    int fam_base; // delta of a member with `e` units is fam_base + e
    int units;    // units of the target
};
__host__ __device__ inline Family family_of(int delta, int M) {
    Family f;
    if (delta >= M) { f.fam_base = M - 2; f.units = delta - (M - 2); }        // A(a), a >= 2
    else            { f.fam_base = -1;    f.units = delta < M - 1 ? delta + 1 : M; } // one node
    return f;
}

// Left-half unit counts m for which both children (s, m) and (S'-s, units-m) exist:
// the closed range [lo, hi] (empty when lo > hi).
__host__ __device__ inline void m_range(int fam_base, int units, int s, int r, int M, int *lo,
                                        int *hi) {
    if (fam_base < 0) { // GPUs of one node: child (s, G(m)) needs s <= m
        *lo = imax(1, s);
        *hi = imin(units - 1, units - r);
    } else {            // whole nodes: child (s, A(m)) needs m <= s <= m*M
        *lo = imax(imax(1, (s + M - 1) / M), units - r);
        *hi = imin(imin(units - 1, s), units - (r + M - 1) / M);
    }
}

} // namespace oob
