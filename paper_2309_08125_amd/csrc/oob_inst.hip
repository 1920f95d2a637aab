// Pipeline-instantiation enumeration (Section 4.2.1, Eq. 5 of the Oobleck paper) for gfx950.
//
// Eq. 5 builds lists by concatenation; on the GPU the lists are never built.  Replacing every
// list by its length turns the equation into a counting recurrence, and the position of a
// vector inside X(p, N') then determines the vector: at (p', N') a position below
// |X(p'-1, N')| lies in the copied part (x_{p'-1} is final), any other position lies in the
// theta part (one more pipeline of size n_{p'-1}, continue at N' - n_{p'-1}).  The paper's
// second requirement (at least f+1 pipelines) filters the final list without reordering it;
// carrying "q more pipelines are still required" as a third index of the count table makes the
// filtered lists directly addressable:
//     C(p', N', q) = C(p'-1, N', q) + C(p', N' - n_{p'-1}, max(q-1, 0)),   C(0, 0, 0) = 1.
// Every output vector is then produced by one lane, independently of all others, and stored
// structure-of-arrays so that a wave writes 128 contiguous bytes per template.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "oob_inst.h"
#include "oob_plan.h"

namespace oob_inst {

constexpr long long kSat = 1ll << 62; // counts saturate here; a saturated total is an error

struct Spec {
    const int *sizes; // may be null: consecutive from n0
    int p, n0, N_lo, N_hi, Q; // Q = f + 1
    long long *cnt;           // [(p+1)][(N_hi+1)][(Q+1)]
};

__device__ __forceinline__ int size_of(const Spec &s, int j) { return s.sizes ? s.sizes[j] : s.n0 + j; }
__device__ __forceinline__ long long cnt_index(const Spec &s, int j, int N, int q) {
    return ((long long)j * (s.N_hi + 1) + N) * (s.Q + 1) + q;
}
__device__ __forceinline__ long long sat_add(long long a, long long b) {
    const unsigned long long c = (unsigned long long)a + (unsigned long long)b; // both <= 2^62: fits 64 bits
    return c > (unsigned long long)kSat ? kSat : (long long)c;
}

// One workgroup.  Plane j of the table needs plane j-1 only, and inside a plane the recurrence
// along N' unrolls into a sum over the number i of size-n pipelines:
//     C(j, N', q) = sum_{i >= 0, i n <= N'} C(j-1, N' - i n, max(q - i, 0)),
// so all entries of a plane are independent: one barrier per template size.
__global__ void __launch_bounds__(1024) k_inst_count(Spec s, long long capacity, long long *offsets, int *status) {
    __shared__ int s_bad;
    __shared__ long long s_tot[OOB_INST_MAX_N + 2];
    const int plane = (s.N_hi + 1) * (s.Q + 1);
    if (threadIdx.x == 0) s_bad = 0;
    __syncthreads();
    for (int j = threadIdx.x; j < s.p; j += blockDim.x) {
        const int n = size_of(s, j);
        if (n < 1 || (j > 0 && n <= size_of(s, j - 1))) s_bad = 1;
    }
    for (int e = threadIdx.x; e < plane; e += blockDim.x) s.cnt[e] = e == 0 ? 1 : 0; // C(0, ., .)
    __syncthreads();
    if (s_bad) { // uniform: every thread leaves here
        for (int i = threadIdx.x; i <= s.N_hi - s.N_lo + 1; i += blockDim.x) offsets[i] = 0;
        if (threadIdx.x == 0) *status = OOB_EINVAL;
        return;
    }
    for (int j = 1; j <= s.p; ++j) {
        const int n = size_of(s, j - 1);
        const long long *prev = s.cnt + (long long)(j - 1) * plane;
        long long *cur = s.cnt + (long long)j * plane;
        for (int e = threadIdx.x; e < plane; e += blockDim.x) {
            const int N = e / (s.Q + 1), q = e - N * (s.Q + 1);
            long long sum = 0;
            for (int i = 0, Ni = N; Ni >= 0; ++i, Ni -= n) {
                const int qi = q - i > 0 ? q - i : 0;
                sum = sat_add(sum, prev[Ni * (s.Q + 1) + qi]);
            }
            cur[e] = sum;
        }
        __syncthreads(); // plane j complete (global memory, same workgroup)
    }
    // exclusive prefix over N' = N_lo..N_hi of the filtered list lengths C(p, N', f+1)
    const int len = s.N_hi - s.N_lo + 1;
    for (int i = threadIdx.x; i < len; i += blockDim.x)
        s_tot[i] = s.cnt[cnt_index(s, s.p, s.N_lo + i, s.Q)];
    __syncthreads();
    if (threadIdx.x == 0) {
        long long run = 0;
        for (int i = 0; i < len; ++i) {
            const long long c = s_tot[i];
            s_tot[i] = run;
            run = sat_add(run, c);
        }
        s_tot[len] = run;
        *status = run >= kSat ? OOB_EOVERFLOW : (capacity >= 0 && run > capacity ? OOB_ECAPACITY : OOB_OK);
    }
    __syncthreads();
    for (int i = threadIdx.x; i <= len; i += blockDim.x) offsets[i] = s_tot[i];
}

// One lane per output vector (grid-stride).  Lanes of a wave hold consecutive list positions,
// which share most of their path through the table: the count loads are mostly broadcasts and
// the stores of one template are 128 contiguous bytes per wave.
__global__ void __launch_bounds__(256) k_inst_unrank(Spec s, const long long *offsets, const int *status,
                                                     unsigned short *x, long long capacity) {
    if (*status != OOB_OK) return;
    const int len = s.N_hi - s.N_lo + 1;
    const long long total = offsets[len];
    const long long stride = (long long)gridDim.x * blockDim.x;
    for (long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += stride) {
        int lo = 0, hi = len - 1; // last N' whose list starts at or before idx
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (offsets[mid] <= idx) lo = mid; else hi = mid - 1;
        }
        int N = s.N_lo + lo, q = s.Q;
        long long rho = idx - offsets[lo];
        for (int j = s.p; j >= 1; --j) {
            const int n = size_of(s, j - 1);
            int xj = 0;
            while (N >= n) { // position inside the copy of X(j-1, N)?  else theta: one more pipeline
                const long long c = s.cnt[cnt_index(s, j - 1, N, q)];
                if (rho < c) break;
                rho -= c;
                ++xj;
                N -= n;
                q = q > 0 ? q - 1 : 0;
            }
            x[(long long)(j - 1) * capacity + idx] = (unsigned short)xj;
        }
    }
}

static bool args_ok(int p, int N_lo, int N_hi, int f) {
    return p >= 1 && p <= OOB_INST_MAX_P && N_lo >= 0 && N_lo <= N_hi && N_hi <= OOB_INST_MAX_N && f >= 0 &&
           f <= OOB_INST_MAX_F;
}

static int run(const int32_t *sizes, int p, int n0, int N_lo, int N_hi, int f, void *ws, size_t ws_bytes,
               uint16_t *x, int64_t capacity, int64_t *offsets, int32_t *status, void *stream, bool enumerate) {
    if (!args_ok(p, N_lo, N_hi, f) || !ws || !offsets || !status) return OOB_EINVAL;
    if (!sizes && n0 < 1) return OOB_EINVAL;
    if (((uintptr_t)ws & 255) != 0) return OOB_EINVAL;
    if (enumerate && (capacity < 0 || (capacity > 0 && !x))) return OOB_EINVAL;
    if (ws_bytes < oob_inst_workspace_size(p, N_hi, f)) return OOB_ECAPACITY;
    Spec s;
    s.sizes = sizes; s.p = p; s.n0 = n0; s.N_lo = N_lo; s.N_hi = N_hi; s.Q = f + 1;
    s.cnt = (long long *)ws;
    hipStream_t st = (hipStream_t)stream;
    hipLaunchKernelGGL(k_inst_count, dim3(1), dim3(1024), 0, st, s, enumerate ? (long long)capacity : -1ll,
                       (long long *)offsets, status);
    if (enumerate && capacity > 0) {
        // enough lanes to keep every CU busy; the kernel strides over the list
        const long long want = (capacity + 255) / 256;
        const int grid = (int)(want < 1 ? 1 : (want > 256 * 16 ? 256 * 16 : want));
        hipLaunchKernelGGL(k_inst_unrank, dim3(grid), dim3(256), 0, st, s, (const long long *)offsets, status,
                           (unsigned short *)x, (long long)capacity);
    }
    return hipGetLastError() == hipSuccess ? OOB_OK : OOB_EHIP;
}

} // namespace oob_inst

extern "C" {

size_t oob_inst_workspace_size(int p, int N_hi, int f) {
    if (!oob_inst::args_ok(p, 0, N_hi, f)) return 0;
    const size_t n = (size_t)(p + 1) * (size_t)(N_hi + 1) * (size_t)(f + 2) * sizeof(long long);
    return (n + 255) & ~(size_t)255;
}

int oob_inst_count(const int32_t *sizes, int p, int n0, int N_lo, int N_hi, int f, void *dev_workspace,
                   size_t workspace_bytes, int64_t *offsets, int32_t *status, void *stream) {
    return oob_inst::run(sizes, p, n0, N_lo, N_hi, f, dev_workspace, workspace_bytes, nullptr, 0, offsets, status,
                         stream, false);
}

int oob_inst_enumerate(const int32_t *sizes, int p, int n0, int N_lo, int N_hi, int f, void *dev_workspace,
                       size_t workspace_bytes, uint16_t *x, int64_t capacity, int64_t *offsets, int32_t *status,
                       void *stream) {
    return oob_inst::run(sizes, p, n0, N_lo, N_hi, f, dev_workspace, workspace_bytes, x, capacity, offsets, status,
                         stream, true);
}

} // extern "C"
