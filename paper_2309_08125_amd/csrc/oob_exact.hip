// Exact minimum of the pipeline cost (Section 4.1.2 of the Oobleck paper; the closed form of
// Eq. 1-4) over all explicit pipelines, for gfx950.
//
// With k* the first slowest stage and tau its time,
//     C = sum_{i<k*} t_i + N_b tau + sum_{i>k*} (2 t_i - tau),
// so around a FIXED slowest stage (u, v, d) the stages before and after it are two independent
// shortest-path problems over (layer, GPUs used):
//     Pre[p][D] = least sum of t over sequences covering layers [0, p) on exactly the first D GPUs, t < tau
//     Suf[p][E] = least sum of (2 t - tau) over sequences covering [p, L) on exactly the last E GPUs, t <= tau
// (no stage crosses a node boundary; boundaries are the multiples of M from either end), and
//     C(u, v, d; n) = min over D of  Pre[u][D] + N_b tau + Suf[v][n M - D - d].
// One workgroup takes one candidate slowest stage at a time (a grid-stride loop over all of
// them), keeps its two tables in its own slice of the workspace (they stay in L2), walks the
// layers with one barrier per layer, each thread owning GPU positions, and merges its minima per
// template into LDS and, at the end, into the result with 64-bit atomic minima.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

#include "oob_exact.h"

namespace oob_exact {

constexpr int kThreads = 256;
constexpr int kSlots = 2048;                    // workgroups in flight (8 waves per SIMD), each with tables of its own
constexpr long long kInf = 1ll << 61;
constexpr long long kForbidden = 1ll << 62;

struct Args {
    oob_profile prof;
    int L, M, n_min, n_max, Nb, Dmax;
    long long cap;
    long long *t;     // [(u (L+1) + v) M + d-1] stage times, -1: impossible
    long long *slots; // [kSlots][2][(L+1)][(Dmax+1)]
    long long *best;
    int *status;
};

inline size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }
inline size_t table_bytes(int L, int M) { return align_up(sizeof(long long) * (size_t)(L + 1) * (L + 1) * M); }
inline size_t slot_bytes(int L, int Dmax) { return align_up(sizeof(long long) * 2 * (size_t)(L + 1) * (Dmax + 1)); }

// Clears the result and validates the magnitudes: every cost is at most (N_b + 2) w, w = the sum
// over the layers of the slowest allowed F + B of the layer plus its boundary term (a bound on the
// sum of all stage times of any pipeline).  status = OOB_EOVERFLOW unless that stays below 2^61.
// One workgroup; runs before k_exact_stages, which only ever lowers the status.
__global__ void __launch_bounds__(kThreads) k_exact_init(Args a) {
    __shared__ long long s_sum[kThreads];
    const int count = a.n_max - a.n_min + 1;
    for (int i = threadIdx.x; i < count; i += kThreads) a.best[i] = kInf;
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
        *a.status = w >= kInf / ((long long)a.Nb + 2) ? OOB_EOVERFLOW : OOB_OK;
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
        a.t[((size_t)u * (a.L + 1) + v) * a.M + d - 1] = val;
    }
    if (bad) atomicExch(a.status, OOB_EINVAL);
}

__global__ void __launch_bounds__(kThreads) k_exact(Args a) {
    HIP_DYNAMIC_SHARED(long long, s_dyn) // [L * M] stage times into (or out of) the current layer, then [count] minima
    const int L = a.L, M = a.M, W = a.Dmax + 1, count = a.n_max - a.n_min + 1;
    long long *s_col = s_dyn, *s_best = s_dyn + (size_t)L * M;
    long long *Pre = a.slots + (size_t)blockIdx.x * 2 * (L + 1) * W, *Suf = Pre + (size_t)(L + 1) * W;
    const long long *bnd = (const long long *)a.prof.boundary_ns;
    if (*a.status != OOB_OK) return; // the same for every thread: nothing is computed from a bad profile
    for (int i = threadIdx.x; i < count; i += kThreads) s_best[i] = kInf;
    const long long ncand = (long long)L * (L + 1) / 2 * M;
    for (long long c = blockIdx.x; c < ncand; c += gridDim.x) {
        // candidate c -> (u, v, d): pairs u < v in row order, d fastest
        const int d = (int)(c % M) + 1;
        long long pr = c / M;
        int u = 0;
        while (pr >= L - u) { pr -= L - u; ++u; }
        const int v = u + 1 + (int)pr;
        const long long tau = a.t[((size_t)u * (L + 1) + v) * M + d - 1];
        if (tau < 0) continue; // the same for the whole workgroup
        __syncthreads();       // the tables of the previous candidate are no longer read

        // Pre[p][.] for p = 0..u
        for (int D = threadIdx.x; D < W; D += kThreads) Pre[D] = D == 0 ? 0 : kInf;
        for (int p = 1; p <= u; ++p) {
            __syncthreads(); // row p-1 written; s_col free
            for (int i = threadIdx.x; i < p * M; i += kThreads) // times of the stages [q, p) on dd GPUs
                s_col[i] = a.t[((size_t)(i / M) * (L + 1) + p) * M + i % M];
            __syncthreads();
            for (int D = threadIdx.x; D < W; D += kThreads) {
                long long m = kInf;
                for (int dd = 1; dd <= M && dd <= D; ++dd) {
                    const int D0 = D - dd;
                    if (D0 % M + dd > M) continue; // would cross a node boundary
                    // a stage [q, p) only gets longer and heavier as q goes down: once it is too slow (or
                    // impossible) it stays so, and the loop ends
                    for (int q = p - 1; q >= 0; --q) {
                        const long long tt = s_col[q * M + dd - 1];
                        if (tt < 0 || tt >= tau) break;
                        const long long x = Pre[(size_t)q * W + D0] + tt;
                        m = x < m ? x : m;
                    }
                }
                Pre[(size_t)p * W + D] = m;
            }
        }
        // Suf[p][.] for p = L..v
        __syncthreads();
        for (int E = threadIdx.x; E < W; E += kThreads) Suf[(size_t)L * W + E] = E == 0 ? 0 : kInf;
        for (int p = L - 1; p >= v; --p) {
            __syncthreads();
            for (int i = threadIdx.x; i < (L - p) * M; i += kThreads) // times of the stages [p, p+1+i/M) on dd GPUs
                s_col[i] = a.t[((size_t)p * (L + 1) + p + 1 + i / M) * M + i % M];
            __syncthreads();
            for (int E = threadIdx.x; E < W; E += kThreads) {
                long long m = kInf;
                for (int dd = 1; dd <= M && dd <= E; ++dd) {
                    const int E0 = E - dd;
                    if (E0 % M + dd > M) continue;
                    // [p, w) as w goes up: impossible stays impossible and the time without the boundary
                    // term only grows, so those end the loop.  The time WITH the boundary term does not
                    // grow (the term belongs to the last layer and the model's last stage pays none):
                    // a stage that is only too slow because of it is skipped, not the rest of the run.
                    for (int w = p + 1; w <= L; ++w) {
                        const long long tt = s_col[(w - p - 1) * M + dd - 1];
                        if (tt < 0) break;
                        if (tt > tau) {
                            if (w == L || tt - bnd[w - 1] > tau) break;
                            continue;
                        }
                        const long long x = Suf[(size_t)w * W + E0] + 2 * tt - tau;
                        m = x < m ? x : m;
                    }
                }
                Suf[(size_t)p * W + E] = m;
            }
        }
        __syncthreads();
        // the slowest stage at every place it fits, for every template
        for (int D = threadIdx.x; D + d < W; D += kThreads) {
            if (D % M + d > M) continue;
            const long long pre = Pre[(size_t)u * W + D];
            if (pre >= kInf / 2) continue;
            for (int n = a.n_min; n <= a.n_max; ++n) {
                const int E = n * M - D - d;
                if (E < 0) continue;
                const long long suf = Suf[(size_t)v * W + E];
                if (suf >= kInf / 2) continue;
                const long long tot = pre + (long long)a.Nb * tau + suf;
                if (tot < s_best[n - a.n_min]) atomicMin((unsigned long long *)&s_best[n - a.n_min], (unsigned long long)tot);
            }
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < count; i += kThreads)
        if (s_best[i] < kInf) atomicMin((unsigned long long *)&a.best[i], (unsigned long long)s_best[i]);
}

__global__ void k_exact_finish(long long *best, int count) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count && best[i] >= kInf / 2) best[i] = -1;
}

} // namespace oob_exact

static bool exact_dims_ok(int L, int n_max, int M) {
    return L >= 1 && L <= OOB_EXACT_MAX_L && n_max >= 1 && M >= 1 && M <= OOB_MAX_GPUS &&
           (long long)n_max * M <= OOB_EXACT_MAX_GPUS;
}

extern "C" size_t oob_exact_workspace_size(int L, int n_max, int gpus_per_node) {
    using namespace oob_exact;
    if (!exact_dims_ok(L, n_max, gpus_per_node)) return 0;
    return table_bytes(L, gpus_per_node) + (size_t)kSlots * slot_bytes(L, n_max * gpus_per_node);
}

extern "C" int oob_exact_minimum(const oob_profile *profile, int L, int n_min, int n_max, int gpus_per_node,
                                 int microbatches, int64_t mem_cap, void *dev_workspace, size_t workspace_bytes,
                                 int64_t *best, int32_t *status, void *stream) {
    using namespace oob_exact;
    if (!profile || !profile->fwd_ns || !profile->bwd_ns || !profile->mem_bytes || !profile->boundary_ns) return OOB_EINVAL;
    if (!best || !status || !dev_workspace || ((uintptr_t)dev_workspace & 255) != 0) return OOB_EINVAL;
    if (n_min < 1 || n_min > n_max || mem_cap <= 0 || !exact_dims_ok(L, n_max, gpus_per_node)) return OOB_EINVAL;
    const int M = gpus_per_node, Dmax = n_max * M;
    if (microbatches < (L < Dmax ? L : Dmax)) return OOB_EINVAL; // the limit S <= N_b is not modelled
    if (workspace_bytes < oob_exact_workspace_size(L, n_max, M)) return OOB_ECAPACITY;
    Args a;
    a.prof = *profile; a.L = L; a.M = M; a.n_min = n_min; a.n_max = n_max; a.Nb = microbatches; a.Dmax = Dmax;
    a.cap = mem_cap;
    a.t = (long long *)dev_workspace;
    a.slots = (long long *)((char *)dev_workspace + table_bytes(L, M));
    a.best = (long long *)best; a.status = status;
    hipStream_t st = (hipStream_t)stream;
    const int count = n_max - n_min + 1;
    hipLaunchKernelGGL(k_exact_init, dim3(1), dim3(kThreads), 0, st, a);
    hipLaunchKernelGGL(k_exact_stages, dim3((L * M + 63) / 64), dim3(64), 0, st, a);
    const long long ncand = (long long)L * (L + 1) / 2 * M;
    const unsigned grid = (unsigned)(ncand < kSlots ? ncand : kSlots);
    const size_t lds = sizeof(long long) * ((size_t)L * M + count);
    hipLaunchKernelGGL(k_exact, dim3(grid), dim3(kThreads), lds, st, a);
    hipLaunchKernelGGL(k_exact_finish, dim3((count + 63) / 64), dim3(64), 0, st, (long long *)best, count);
    return hipGetLastError() == hipSuccess ? OOB_OK : OOB_EHIP;
}
