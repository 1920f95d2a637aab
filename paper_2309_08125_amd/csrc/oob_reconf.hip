// Reconfiguration simulator (Section 5.1 and Appendix B of the Oobleck paper) for gfx950.
//
// One lane runs one failure sequence.  A trajectory's state is small (at most 64 pipeline sizes
// and a 64-bit mask of the list positions still in use), but it is indexed by data: the sizes
// live in LDS, one column per lane (sizes[position][lane], 16 bits, as many rows as there are
// starting pipelines), so that the lanes of a wave never share a bank row for the same position,
// and the mask lives in a register pair.  A list position whose pipeline was absorbed keeps size
// 0, so the two loops that run at every step (which pipeline holds the failing node; who can
// lend) walk all positions with a wave-uniform counter and no branch: LDS offsets are the same
// for all lanes and nothing diverges.  Only the rare merge walks the mask.
// Draws are read and trace words written with the trajectory index fastest, so every global
// access of a wave is one contiguous line.  Every loop below ends after at most 64 or `burst`
// rounds for every lane.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "oob_plan.h"
#include "oob_reconf.h"

namespace oob_reconf {

constexpr int kLanes = 256; // trajectories per workgroup
constexpr int kUnroll = 4;  // list positions per round of the two scans; the list is padded with empty ones

struct Args {
    const int *sizes0;
    int c0, n0, n_hi, f;
    const unsigned *draws;
    int steps, burst;
    long long T;
    unsigned *trace;
    int *final_sizes, *summary, *status;
};

// Starting pipelines must be template sizes and few enough nodes for 16 bits.
__device__ __forceinline__ bool start_ok(const Args &a) {
    long long sum = 0;
    for (int i = 0; i < a.c0; ++i) {
        const int s = a.sizes0[i];
        if (s < a.n0 || s > a.n_hi) return false;
        sum += s;
    }
    return sum <= OOB_RECONF_MAX_NODES;
}

__global__ void __launch_bounds__(kLanes) k_reconf(Args a) {
    HIP_DYNAMIC_SHARED(unsigned short, sizes) // [rows][kLanes], rows = c0 rounded up to kUnroll
    const int lane = threadIdx.x;
    const long long t = (long long)blockIdx.x * kLanes + lane;
    const bool ok = start_ok(a);
    if (t == 0) *a.status = ok ? OOB_OK : OOB_EINVAL;
    if (!ok || t >= a.T) return;

    unsigned short *mine = sizes + lane; // position i at mine[i * kLanes]
    const int rows = (a.c0 + kUnroll - 1) / kUnroll * kUnroll;
    unsigned total = 0;
    for (int i = 0; i < rows; ++i) {
        const int s = i < a.c0 ? a.sizes0[i] : 0;
        mine[i * kLanes] = (unsigned short)s;
        total += (unsigned)s;
    }
    unsigned long long alive = a.c0 == 64 ? ~0ull : (1ull << a.c0) - 1;
    const unsigned need = (unsigned)(a.f + 1) * (unsigned)a.n0; // fewer nodes: training stops
    int stop = OOB_RECONF_STOP_NONE, viol = 0;
    int survived = 0, sum_reinst = 0, sum_borrowed = 0, sum_merges = 0;
    const unsigned *step_draws = a.draws + t;              // this step's first draw of this trajectory
    const long long step_stride = (long long)a.burst * a.T;
    unsigned *word = a.trace ? a.trace + t : nullptr;      // this step's trace word

    for (int step = 0; step < a.steps; ++step, step_draws += step_stride) {
        int reinst = 0, borrowed = 0, merges = 0;
        if (stop == OOB_RECONF_STOP_NONE) {
            // the losses of this step
            unsigned long long affected = 0;
            const unsigned *draw = step_draws;
            for (int b = 0; b < a.burst && total > 0; ++b, draw += a.T) {
                const unsigned r = __umulhi(*draw, total); // floor(draw * total / 2^32) < total
                // The pipeline that holds node r is the number of positions whose running sum of
                // sizes is <= r (absorbed and empty positions add nothing).  It is below c0, since
                // the last running sum is total > r.
                unsigned run = 0;
                int hit = 0;
                for (int i = 0; i < rows; i += kUnroll) {
#pragma unroll
                    for (int e = 0; e < kUnroll; ++e) {
                        run += mine[(i + e) * kLanes];
                        hit += run <= r;
                    }
                }
                mine[hit * kLanes] -= 1;
                affected |= 1ull << hit;
                --total;
            }
            if (total < need) {
                stop = OOB_RECONF_STOP_TOO_FEW_NODES;
            } else {
                // repairs, in list order
                while (affected && stop == OOB_RECONF_STOP_NONE) {
                    const int i = __ffsll((long long)affected) - 1;
                    affected &= affected - 1;
                    if (!((alive >> i) & 1)) continue; // absorbed by an earlier repair
                    int si = mine[i * kLanes];
                    if (si >= a.n0) { ++reinst; continue; }
                    while (si < a.n0) { // borrow from the largest pipeline above n0, first of equals
                        // one max over (size, 63 - position); position i itself is below n0 here
                        unsigned best = 0;
                        for (int k = 0; k < rows; k += kUnroll) {
#pragma unroll
                            for (int e = 0; e < kUnroll; ++e) {
                                const unsigned key = (unsigned)mine[(k + e) * kLanes] << 6 | (unsigned)(63 - k - e);
                                best = key > best ? key : best;
                            }
                        }
                        if ((int)(best >> 6) <= a.n0) break;
                        mine[(63 - (int)(best & 63)) * kLanes] = (unsigned short)((best >> 6) - 1);
                        ++si;
                        ++borrowed;
                    }
                    while (si < a.n0) { // absorb the smallest other pipeline, first of equals
                        int best = 1 << 30, j = -1;
                        for (unsigned long long m = alive & ~(1ull << i); m; m &= m - 1) {
                            const int k = __ffsll((long long)m) - 1;
                            const int s = mine[k * kLanes];
                            if (s < best) { best = s; j = k; }
                        }
                        if (j < 0) { stop = OOB_RECONF_STOP_NO_PARTNER; break; }
                        si += best;
                        mine[j * kLanes] = 0;
                        alive &= ~(1ull << j);
                        ++merges;
                    }
                    mine[i * kLanes] = (unsigned short)si;
                    if (stop == OOB_RECONF_STOP_NONE && si > a.n_hi) viol |= 1;
                }
                if (stop == OOB_RECONF_STOP_NONE) {
                    ++survived;
                    if (__popcll(alive) < a.f + 1) viol |= 2;
                }
            }
            sum_reinst += reinst; sum_borrowed += borrowed; sum_merges += merges;
        }
        if (word) {
            *word = (unsigned)reinst | (unsigned)borrowed << 8 | (unsigned)merges << 16 |
                    (unsigned)__popcll(alive) << 23 | (unsigned)stop << 30;
            word += a.T;
        }
    }

    if (a.final_sizes)
        for (int i = 0; i < a.c0; ++i) a.final_sizes[(long long)i * a.T + t] = mine[i * kLanes];
    int *sm = a.summary + t;
    sm[OOB_RECONF_SURVIVED * a.T] = survived;
    sm[OOB_RECONF_REINSTANTIATED * a.T] = sum_reinst;
    sm[OOB_RECONF_BORROWED * a.T] = sum_borrowed;
    sm[OOB_RECONF_MERGES * a.T] = sum_merges;
    sm[OOB_RECONF_ALIVE * a.T] = __popcll(alive);
    sm[OOB_RECONF_NODES * a.T] = (int)total;
    sm[OOB_RECONF_VIOLATIONS * a.T] = viol;
    sm[OOB_RECONF_STOP * a.T] = stop;
}

} // namespace oob_reconf

extern "C" int oob_reconf_simulate(const int32_t *sizes0, int c0, int n0, int n_hi, int f,
                                   const uint32_t *draws, int steps, int burst, int64_t T,
                                   uint32_t *trace, int32_t *final_sizes, int32_t *summary,
                                   int32_t *status, void *stream) {
    using namespace oob_reconf;
    if (!sizes0 || !summary || !status) return OOB_EINVAL;
    if (c0 < 1 || c0 > OOB_RECONF_MAX_PIPELINES || n0 < 1 || n_hi < n0 || n_hi > OOB_RECONF_MAX_NODES || f < 0)
        return OOB_EINVAL;
    if ((long long)(f + 1) * n0 > OOB_RECONF_MAX_NODES) return OOB_EINVAL;
    if (steps < 0 || burst < 1 || burst > OOB_RECONF_MAX_BURST || T < 1) return OOB_EINVAL;
    if (steps > 0 && !draws) return OOB_EINVAL;
    const long long blocks = (T + kLanes - 1) / kLanes;
    if (blocks > 0x7fffffffll) return OOB_EINVAL;
    Args a;
    a.sizes0 = sizes0; a.c0 = c0; a.n0 = n0; a.n_hi = n_hi; a.f = f;
    a.draws = draws; a.steps = steps; a.burst = burst; a.T = T;
    a.trace = trace; a.final_sizes = final_sizes; a.summary = summary; a.status = status;
    const size_t lds = (size_t)((c0 + kUnroll - 1) / kUnroll * kUnroll) * kLanes * sizeof(unsigned short); // <= 32 KB
    hipLaunchKernelGGL(k_reconf, dim3((unsigned)blocks), dim3(kLanes), lds, (hipStream_t)stream, a);
    return hipGetLastError() == hipSuccess ? OOB_OK : OOB_EHIP;
}
