// Table layout and index arithmetic shared by the host driver and the kernels.
//
// Notation (Section 4.1.2 of the paper): a state is (S', u, v, delta): layers [u, v) cut into
// S' stages on device set delta.  Device sets: G(g) = g GPUs inside one node (delta = g-1,
// 1 <= g <= M-1) and A(a) = a whole nodes (delta = M-2+a).  Both kinds form an additive
// family: a set of `units` is split into m and units-m, with delta = fam_base + units where
// fam_base = -1 inside a node (units = GPUs; A(1) counts as M GPUs when it is the target)
// and fam_base = M-2 across nodes (units = nodes).
//
// Storage.  Every valid (S', delta) owns one table: the (u, v) plane in ABSOLUTE layer
// coordinates, 0 <= u <= v <= L, cut into 8 x 8 blocks: block row u/8, block column (v + c)/8
// with the column shift c = col_shift(L), which puts v = L into the last column of its block
// (only block columns >= block rows are kept), 64 records per block, row-major inside the block.
// The shift matters because the states that end at the last layers are the ones every level needs
// and a ragged last block column would leave most of its lanes idle; the ragged column is the
// first one instead (v < 0, no states).  Rows need no shift: u = 0 already starts a block.
// Absolute coordinates make the three operands of a split at k line up on the same block
// grid: left child at (u, k), right child at (k, v), target at (u, v) -- the layout of a
// blocked matrix product (a split point k is column k + c of the left child's table and row k of
// the right child's).  Entries that are not states (v - u < S', u >= L, v < 0) inside a
// block that holds at least one state carry the "no such state" value, so inner loops need
// no masks; blocks without any state are never written and never read.
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
__host__ __device__ inline int cdiv(int a, int b) { return (a + b - 1) / b; }

// (S', delta) exists ("Choosing the number of stages": a stage never spans nodes and every
// GPU is used): G(g): S' <= g;  A(a): a <= S' <= a*M.  The valid deltas of a level are the
// contiguous range [dlo, dhi].
__host__ __device__ inline int dlo_of(int S, int M) { return S <= M ? S - 1 : M - 2 + cdiv(S, M); }
__host__ __device__ inline int dhi_of(int S, int M, int n_max) { return M - 2 + imin(S, n_max); }

__host__ __device__ inline int smax_of(int L, int n_max, int M, int Nb) {
    long long s = L;
    if ((long long)n_max * M < s) s = (long long)n_max * M;
    if (Nb > 0 && Nb < s) s = Nb;
    return (int)s;
}

// Family of a target device set.
struct Family {
    int fam;      // 0: inside one node (units = GPUs), 1: across nodes (units = nodes)
    int fam_base; // delta of a member with `e` units is fam_base + e
    int units;    // units of the target
};
__host__ __device__ inline Family family_of(int delta, int M) {
    Family f;
    if (delta >= M) { f.fam = 1; f.fam_base = M - 2; f.units = delta - (M - 2); }               // A(a), a >= 2
    else            { f.fam = 0; f.fam_base = -1;    f.units = delta < M - 1 ? delta + 1 : M; } // one node
    return f;
}

// Unit counts e for which the CHILD state (S, member e of the family) exists: [lo, hi].
// Across nodes: ceil(S/M) <= e <= min(S, n_max).  Inside a node a child is always some
// G(e): S <= e <= M-1.
__host__ __device__ inline void child_units(int fam, int S, int M, int n_max, int *lo, int *hi) {
    if (fam == 0) { *lo = S; *hi = M - 1; }
    else              { *lo = cdiv(S, M); *hi = imin(S, n_max); }
}

// Left-half unit counts m for which both children (s, m) and (r, units-m) exist: [lo, hi]
// (empty when lo > hi).
__host__ __device__ inline void m_range(int fam, int units, int s, int r, int M, int n_max,
                                        int *lo, int *hi) {
    int alo, ahi, blo, bhi;
    child_units(fam, s, M, n_max, &alo, &ahi);
    child_units(fam, r, M, n_max, &blo, &bhi);
    *lo = imax(alo, units - bhi);
    *hi = imin(ahi, units - blo);
}

// Target unit counts of a family at level S': inside a node S' <= g <= M (g = M is A(1));
// across nodes max(2, ceil(S'/M)) <= a <= min(S', n_max).
__host__ __device__ inline void target_units(int fam, int S, int M, int n_max, int *lo, int *hi) {
    if (fam == 0) { *lo = S; *hi = M; }
    else          { *lo = imax(2, cdiv(S, M)); *hi = imin(S, n_max); }
}

// Bits that hold a split point k <= L.
__host__ __device__ inline int key_bits(int L) {
    int b = 1;
    while ((1 << b) <= L) ++b;
    return b;
}

// ---- blocked (u, v) plane ----------------------------------------------------------------
__host__ __device__ inline int nblocks_of(int L) { return L / 8 + 1; } // v runs 0..L
__host__ __device__ inline int col_shift(int L) { return (8 - ((L + 1) & 7)) & 7; }
__host__ __device__ inline int tri_blocks(int NB) { return NB * (NB + 1) / 2; }
__host__ __device__ inline int tri_index(int ub, int vb, int NB) {
    return ub * NB - ub * (ub - 1) / 2 + (vb - ub);
}
// Record of (u, v) inside a table (c = col_shift(L)).
__host__ __device__ inline int rec_off(int u, int v, int c, int NB) {
    return tri_index(u >> 3, (v + c) >> 3, NB) * 64 + ((u & 7) << 3) + ((v + c) & 7);
}

// Blocks of level S' that hold at least one state: (ub, vb = ub + d) with 8 d + 7 - c >= S' and
// 8 ub + S' <= L.  They are enumerated by decreasing d (the blocks far from the diagonal have
// the longest split ranges, so the heaviest workgroups start first).
__host__ __device__ inline int tile_dmin(int L, int S) { return (S + col_shift(L)) / 8; } // = ceil((S' + c - 7) / 8)
__host__ __device__ inline int tile_count(int L, int S) {
    const int NB = nblocks_of(L), ubmax = (L - S) / 8;
    int c = 0;
    for (int d = NB - 1; d >= tile_dmin(L, S); --d) c += imin(ubmax, NB - 1 - d) + 1;
    return c;
}
__host__ __device__ inline void tile_decode(int L, int S, int t, int *ub, int *vb) {
    const int NB = nblocks_of(L), ubmax = (L - S) / 8;
    for (int d = NB - 1; d >= tile_dmin(L, S); --d) {
        const int c = imin(ubmax, NB - 1 - d) + 1;
        if (t < c) { *ub = t; *vb = t + d; return; }
        t -= c;
    }
    *ub = 0; *vb = 0;
}
// Last layer position of block column vb (the last block column ends at L exactly).
__host__ __device__ inline int tile_vmax(int L, int vb) { return vb * 8 + 7 - col_shift(L); }

// Split points k of a block of the plane at level S': kmin = 8 ub + s .. kmax = vmax - (S' - s):
// their number does not depend on s.  The keyed split kernel cuts this range into segments of
// about seg_target() consecutive k, one workgroup each: as many segments as the range divided by
// the target gives, rounded to the nearest (at least one), all of the same length up to one
// split point -- so no workgroup is left with a stub of one or two split points, which would pay
// the whole set-up and the merge of its keys for next to nothing.
constexpr int kSegTarget = 8, kSegTargetTop = 3, kSegTopLayers = 28; // measured on the headline workload
constexpr int kSegMin = 3; // no target below this (sizes the task lists)
// The top levels (fewer than kSegTopLayers layers of slack, a handful of blocks) cannot fill the
// machine with workgroups of eight split points: there the target is three.
__host__ __device__ inline int seg_target(int L, int S) { return L - S < kSegTopLayers ? kSegTargetTop : kSegTarget; }
__host__ __device__ inline int tile_krange(int L, int S, int ub, int vb) {
    return tile_vmax(L, vb) - ub * 8 - S + 1;
}
__host__ __device__ inline int seg_n(int krange, int target) { return imax(1, (krange + target / 2) / target); }
// Segment j of n over a range of `krange` split points: offset of its first one and its length.
__host__ __device__ inline void seg_span(int krange, int n, int j, int *ofs, int *len) {
    const int base = krange / n, extra = krange % n;
    *ofs = j * base + imin(j, extra);
    *len = base + (j < extra ? 1 : 0);
}
__host__ __device__ inline int seg_count(int L, int S) { // over all blocks of the level
    const int NB = nblocks_of(L), ubmax = (L - S) / 8;
    int c = 0;
    for (int d = NB - 1; d >= tile_dmin(L, S); --d)
        for (int ub = 0; ub <= imin(ubmax, NB - 1 - d); ++ub) c += seg_n(tile_krange(L, S, ub, ub + d), seg_target(L, S));
    return c;
}
// Upper bounds that grow with L, for sizing a workspace that serves every L up to a maximum: the
// counts of the same plane without the column shift (a shifted plane never has more blocks of a
// level), with every split range cut at the smallest segment target.
__host__ __device__ inline int tile_count_bound(int L, int S) {
    const int NB = nblocks_of(L), ubmax = (L - S) / 8;
    int c = 0;
    for (int d = NB - 1; d >= S / 8; --d) c += imin(ubmax, NB - 1 - d) + 1;
    return c;
}
__host__ __device__ inline int seg_count_bound(int L) {
    const int NB = nblocks_of(L), ubmax = (L - 2) / 8;
    int c = 0;
    for (int d = NB - 1; d >= 0; --d)
        for (int ub = 0; ub <= imin(ubmax, NB - 1 - d); ++ub)
            c += cdiv(imin((ub + d) * 8 + 7, L) - ub * 8 - 2 + 1, kSegMin) + 1;
    return c;
}

} // namespace oob
