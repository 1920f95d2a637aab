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
#include <stdlib.h>

#include <atomic>
#include <mutex>
#include <type_traits>

#include "oob_inst.h"
#include "oob_plan.h"

namespace oob_inst {

constexpr long long kSat = 1ll << 62; // counts saturate here; a saturated total is an error
constexpr int kGroup = 8;             // counts a lane reads at once

// Count table: row (N', q) holds C(j, N', q) for j = 0..p, padded to whole groups, so that the
// counts a position is compared with (same N', same q, descending j) are contiguous.
struct Spec {
    const int *sizes; // may be null: consecutive from n0
    int p, n0, N_lo, N_hi, Q, R; // Q = f + 1; R = row length
    long long *cnt;              // [(N_hi+1)][(Q+1)][R]
    unsigned *cnt32;             // the same table in 32 bits, valid if *narrow
    int *narrow;                 // [1] every count is below 2^32
};
constexpr size_t kHeaderBytes = 256; // the workspace starts with `narrow`, the two tables follow

__host__ __device__ inline int row_len(int p) { return (p + 1 + kGroup - 1) / kGroup * kGroup; }
__device__ __forceinline__ int size_of(const Spec &s, int j) { return s.sizes ? s.sizes[j] : s.n0 + j; }
__device__ __forceinline__ long long sat_add(long long a, long long b) {
    const unsigned long long c = (unsigned long long)a + (unsigned long long)b; // both <= 2^62: fits 64 bits
    return c > (unsigned long long)kSat ? kSat : (long long)c;
}

// One workgroup.  Plane j of the table (all N', q) needs plane j-1 only, and inside a plane the
// recurrence along N' unrolls into a sum over the number i of size-n pipelines:
//     C(j, N', q) = sum_{i >= 0, i n <= N'} C(j-1, N' - i n, max(q - i, 0)),
// so all entries of a plane are independent: one barrier per template size.  With IN_LDS the
// previous and the current plane live in LDS (two planes of (N_hi+1)(Q+1) counts); otherwise
// the previous plane is read back from the table.
template <bool IN_LDS>
__global__ void __launch_bounds__(1024) k_inst_count(Spec s, long long *offsets, int *status, int keep_wide) {
    HIP_DYNAMIC_SHARED(long long, s_dyn) // IN_LDS: two planes; then reused for the prefix sum
    __shared__ int s_bad;
    __shared__ unsigned long long s_max;
    const int QQ = s.Q + 1, plane = (s.N_hi + 1) * QQ, len = s.N_hi - s.N_lo + 1;
    if (threadIdx.x == 0) { s_bad = 0; s_max = 0; }
    __syncthreads();
    for (int j = threadIdx.x; j < s.p; j += blockDim.x) {
        const int n = size_of(s, j);
        if (n < 1 || (j > 0 && n <= size_of(s, j - 1))) s_bad = 1;
    }
    for (int e = threadIdx.x; e < plane; e += blockDim.x) { // C(0, ., .)
        const long long c = e == 0 ? 1 : 0;
        s.cnt[(long long)e * s.R] = c;
        if (IN_LDS) s_dyn[e] = c;
        // the padding of a row compares greater than any list position
        for (int j = s.p + 1; j < s.R; ++j) s.cnt[(long long)e * s.R + j] = 0x7FFFFFFFFFFFFFFFll;
    }
    __syncthreads();
    if (s_bad) { // uniform: every thread leaves here
        for (int i = threadIdx.x; i <= len; i += blockDim.x) offsets[i] = 0;
        if (threadIdx.x == 0) { *status = OOB_EINVAL; *s.narrow = 0; }
        return;
    }
    long long mine = 1; // largest count this thread has written
    for (int j = 1; j <= s.p; ++j) {
        const int n = size_of(s, j - 1);
        const long long *prev = IN_LDS ? s_dyn + ((j - 1) & 1) * plane : s.cnt + (j - 1);
        const long long pstride = IN_LDS ? 1 : s.R;
        long long *cur = s_dyn + (j & 1) * plane;
        for (int e = threadIdx.x; e < plane; e += blockDim.x) {
            const int N = e / QQ, q = e - N * QQ;
            long long sum = 0;
            for (int i = 0, Ni = N; Ni >= 0; ++i, Ni -= n) {
                const int qi = q - i > 0 ? q - i : 0;
                sum = sat_add(sum, prev[(long long)(Ni * QQ + qi) * pstride]);
            }
            s.cnt[(long long)e * s.R + j] = sum;
            if (IN_LDS) cur[e] = sum;
            mine = sum > mine ? sum : mine;
        }
        __syncthreads(); // plane j complete (LDS, or global memory written by this workgroup)
    }
    // exclusive prefix over N' = N_lo..N_hi of the filtered list lengths C(p, N', f+1)
    for (int i = threadIdx.x; i < len; i += blockDim.x)
        s_dyn[i] = s.cnt[((long long)(s.N_lo + i) * QQ + s.Q) * s.R + s.p];
    __syncthreads();
    if (threadIdx.x == 0) {
        long long run = 0;
        for (int i = 0; i < len; ++i) {
            const long long c = s_dyn[i];
            s_dyn[i] = run;
            run = sat_add(run, c);
        }
        s_dyn[len] = run;
        *status = run >= kSat ? OOB_EOVERFLOW : OOB_OK;
    }
    __syncthreads();
    for (int i = threadIdx.x; i <= len; i += blockDim.x) offsets[i] = s_dyn[i];
    // While every count is below 2^32 a second copy of the table in 32 bits halves what a lane
    // reads per comparison step (the reads bound the enumeration kernel); padding stays maximal.
    atomicMax(&s_max, (unsigned long long)mine);
    __syncthreads();
    const bool narrow = s_max < (1ull << 32) && !keep_wide;
    if (narrow)
        for (long long e = threadIdx.x; e < (long long)plane * s.R; e += blockDim.x) {
            const long long v = s.cnt[e];
            s.cnt32[e] = v == 0x7FFFFFFFFFFFFFFFll ? 0xFFFFFFFFu : (unsigned)v;
        }
    if (threadIdx.x == 0) *s.narrow = narrow;
}

// One lane per output vector (grid-stride).  A vector at position rho of the list of (N', q)
// over the first j sizes has its highest non-zero count at the largest i < j with
// C(i, N', q) <= rho (the lists over fewer sizes are prefixes of the list over more); it then
// continues at position rho - C(i, N', q) of (N' - n_i, q - 1) over the first i+1 sizes.  The
// sizes are visited in groups of kGroup from the top: all lanes take the same trip through
// the groups, so the kGroup counts of a group are stored by whole waves (128 contiguous bytes
// per template), and one read of kGroup counts fetches every count a lane must compare with in
// that group.  C is non-decreasing along a row, so the number of entries <= rho locates i without
// a search, and a group whose first count exceeds rho holds no pipeline of this vector.
template <typename CT> // long long, or unsigned when the counting kernel could narrow the table
__device__ __forceinline__ void unrank_all(const Spec &s, const long long *offsets, unsigned short *x,
                                           long long capacity, long long total) {
    const int len = s.N_hi - s.N_lo + 1, QQ = s.Q + 1;
    const long long stride = (long long)gridDim.x * blockDim.x;
    const CT *tab = sizeof(CT) == 4 ? (const CT *)s.cnt32 : (const CT *)s.cnt;
    for (long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += stride) {
        int lo = 0, hi = len - 1; // last N' whose list starts at or before idx
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (offsets[mid] <= idx) lo = mid; else hi = mid - 1;
        }
        int N = s.N_lo + lo, q = s.Q;
        CT rho = (CT)(idx - offsets[lo]);
        // A group can hold a pipeline only if its first count is <= rho.  The first counts of up to
        // eight groups are read in one go (independent reads), so that the many empty groups of the
        // large sizes cost one round trip together instead of one each.
        int gcov = (s.p - 1) / kGroup + 1; // groups gcov.. have been probed with the current (N, q, rho)
        int gnext = -1;                    // highest probed group that can hold a pipeline
        for (int g = (s.p - 1) / kGroup; g >= 0; --g) {
            const int base = g * kGroup;
            if (g < gcov) {
                const CT *r0 = tab + ((long long)N * QQ + q) * s.R;
                CT f[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) f[i] = r0[(g - i > 0 ? g - i : 0) * kGroup];
                gnext = -1;
#pragma unroll
                for (int i = 7; i >= 0; --i)
                    if (g - i >= 0 && f[i] <= rho) gnext = g - i;
                gcov = g - 7 > 0 ? g - 7 : 0;
            }
            int kcap = s.p - 1 - base < kGroup - 1 ? s.p - 1 - base : kGroup - 1; // sizes base..base+kcap may get a pipeline
            unsigned long long xlo = 0, xhi = 0; // kGroup 16-bit counts
            while (g == gnext) {
                const CT *row = tab + ((long long)N * QQ + q) * s.R + base;
                CT c[kGroup];
#pragma unroll
                for (int k = 0; k < kGroup; ++k) c[k] = row[k];
                gcov = g;              // whatever follows changes (N, q, rho): the groups below are probed again
                if (c[0] > rho) break; // nothing (more) in this group
                int m = 0;             // entries <= rho: a prefix of the row
#pragma unroll
                for (int k = 0; k < kGroup; ++k) m += c[k] <= rho ? 1 : 0;
                const int ks = m - 1 < kcap ? m - 1 : kcap;
                // c[ks] by halving (no indexed registers)
                const bool b0 = ks & 1, b1 = ks & 2, b2 = ks & 4;
                const CT c01 = b0 ? c[1] : c[0], c23 = b0 ? c[3] : c[2], c45 = b0 ? c[5] : c[4], c67 = b0 ? c[7] : c[6];
                const CT c03 = b1 ? c23 : c01, c47 = b1 ? c67 : c45;
                const CT ck = b2 ? c47 : c03;
                const int nk = size_of(s, base + ks); // consecutive sizes: arithmetic; a list: one cached read
                if (nk > N) break; // cannot happen with a consistent table; keeps the loop finite
                rho -= ck;
                N -= nk;
                q = q > 0 ? q - 1 : 0;
                kcap = ks;
                const unsigned long long one = 1ull << (16 * (ks & 3));
                if (b2) xhi += one; else xlo += one;
            }
            unsigned short *xr = x + (long long)base * capacity + idx; // row `base` of the output, this lane's column
            if (base + kGroup <= s.p) { // whole group: no per-template test
#pragma unroll
                for (int k = 0; k < kGroup; ++k, xr += capacity)
                    *xr = (unsigned short)((k < 4 ? xlo : xhi) >> (16 * (k & 3)));
            } else {
#pragma unroll
                for (int k = 0; k < kGroup; ++k, xr += capacity)
                    if (base + k < s.p) *xr = (unsigned short)((k < 4 ? xlo : xhi) >> (16 * (k & 3)));
            }
        }
    }
}

__global__ void __launch_bounds__(256) k_inst_unrank(Spec s, const long long *offsets, int *status,
                                                     unsigned short *x, long long capacity) {
    if (*status != OOB_OK) return;
    const long long total = offsets[s.N_hi - s.N_lo + 1];
    if (total > capacity) { // uniform: nothing is written
        if (blockIdx.x == 0 && threadIdx.x == 0) *status = OOB_ECAPACITY;
        return;
    }
    if (*s.narrow) unrank_all<unsigned>(s, offsets, x, capacity, total); // the table's type is known here only
    else unrank_all<long long>(s, offsets, x, capacity, total);
}

static bool args_ok(int p, int N_lo, int N_hi, int f) {
    return p >= 1 && p <= OOB_INST_MAX_P && N_lo >= 0 && N_lo <= N_hi && N_hi <= OOB_INST_MAX_N && f >= 0 &&
           f <= OOB_INST_MAX_F;
}

static size_t wide_bytes(int p, int N_hi, int f) {
    const size_t n = (size_t)(N_hi + 1) * (size_t)(f + 2) * (size_t)row_len(p) * sizeof(long long);
    return (n + 255) & ~(size_t)255;
}
static size_t table_bytes(int p, int N_hi, int f) { // header, 64-bit table, 32-bit table
    return kHeaderBytes + wide_bytes(p, N_hi, f) + wide_bytes(p, N_hi, f) / 2 + 256;
}

static int check_spec(const int32_t *sizes, int p, int n0, int N_lo, int N_hi, int f, void *ws, size_t ws_bytes,
                      int64_t *offsets, int32_t *status, Spec *s) {
    if (!args_ok(p, N_lo, N_hi, f) || !ws || !offsets || !status) return OOB_EINVAL;
    if (!sizes && n0 < 1) return OOB_EINVAL;
    if (((uintptr_t)ws & 255) != 0) return OOB_EINVAL;
    if (ws_bytes < table_bytes(p, N_hi, f)) return OOB_ECAPACITY;
    s->sizes = sizes; s->p = p; s->n0 = n0; s->N_lo = N_lo; s->N_hi = N_hi; s->Q = f + 1;
    s->R = row_len(p);
    s->narrow = (int *)ws;
    s->cnt = (long long *)((char *)ws + kHeaderBytes);
    s->cnt32 = (unsigned *)((char *)ws + kHeaderBytes + wide_bytes(p, N_hi, f));
    return OOB_OK;
}

static std::atomic<int> g_keep_wide{0}; // test hook: never use the 32-bit copy of the table

static int launch_count(const Spec &s, int64_t *offsets, int32_t *status, hipStream_t stream) {
    const int keep_wide = g_keep_wide.load();
    const size_t plane = (size_t)(s.N_hi + 1) * (s.Q + 1) * sizeof(long long);
    const size_t scan = (size_t)(s.N_hi - s.N_lo + 2) * sizeof(long long);
    if (2 * plane <= 128 * 1024) {
        const size_t lds = 2 * plane > scan ? 2 * plane : scan;
        if (lds > 64 * 1024 &&
            hipFuncSetAttribute((const void *)k_inst_count<true>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds) != hipSuccess)
            return OOB_EHIP;
        hipLaunchKernelGGL(k_inst_count<true>, dim3(1), dim3(1024), lds, stream, s, (long long *)offsets, status,
                           keep_wide);
    } else {
        hipLaunchKernelGGL(k_inst_count<false>, dim3(1), dim3(1024), scan, stream, s, (long long *)offsets, status,
                           keep_wide);
    }
    return hipGetLastError() == hipSuccess ? OOB_OK : OOB_EHIP;
}

static int launch_unrank(const Spec &s, const int64_t *offsets, int32_t *status, uint16_t *x, int64_t capacity,
                         hipStream_t stream) {
    // one lane per vector of the capacity; the kernel strides if the grid limit cuts that short
    const long long want = (capacity + 255) / 256;
    const int grid = (int)(want < 1 ? 1 : (want > (1 << 22) ? (1 << 22) : want));
    hipLaunchKernelGGL(k_inst_unrank, dim3(grid), dim3(256), 0, stream, s, (const long long *)offsets, status,
                       (unsigned short *)x, (long long)capacity);
    return hipGetLastError() == hipSuccess ? OOB_OK : OOB_EHIP;
}

// The count table of oob_inst_enumerate_static: one array per GPU, part of the loaded code object
// (so nothing is ever allocated for it), held until the process ends.  `scratch` itself is a
// host-side stand-in, not a device address: host code uses the address hipGetSymbolAddress reports
// for the current device, looked up once per device.
static __device__ __align__(256) unsigned char scratch[OOB_INST_STATIC_BYTES];
constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mu;
static void *g_scratch_ptr[kMaxDevices];

static int static_table(void **ws) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return OOB_EHIP;
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return OOB_EHIP;
        }
        g_scratch_ptr[dev] = ptr;
    }
    *ws = g_scratch_ptr[dev];
    return OOB_OK;
}

} // namespace oob_inst

extern "C" {

int oob_inst_keep_wide_table(int on) { return oob_inst::g_keep_wide.exchange(on != 0); }

size_t oob_inst_workspace_size(int p, int N_hi, int f) {
    if (!oob_inst::args_ok(p, 0, N_hi, f)) return 0;
    return oob_inst::table_bytes(p, N_hi, f);
}

int oob_inst_count(const int32_t *sizes, int p, int n0, int N_lo, int N_hi, int f, void *dev_workspace,
                   size_t workspace_bytes, int64_t *offsets, int32_t *status, void *stream) {
    using namespace oob_inst;
    Spec s;
    const int rc = check_spec(sizes, p, n0, N_lo, N_hi, f, dev_workspace, workspace_bytes, offsets, status, &s);
    if (rc != OOB_OK) return rc;
    return launch_count(s, offsets, status, (hipStream_t)stream);
}

int oob_inst_enumerate(const int32_t *sizes, int p, int n0, int N_lo, int N_hi, int f, void *dev_workspace,
                       size_t workspace_bytes, uint16_t *x, int64_t capacity, const int64_t *offsets,
                       int32_t *status, void *stream) {
    using namespace oob_inst;
    Spec s;
    const int rc = check_spec(sizes, p, n0, N_lo, N_hi, f, dev_workspace, workspace_bytes, (int64_t *)offsets,
                              status, &s);
    if (rc != OOB_OK) return rc;
    if (capacity < 0 || (capacity > 0 && !x)) return OOB_EINVAL;
    return launch_unrank(s, offsets, status, x, capacity, (hipStream_t)stream);
}

int oob_inst_enumerate_static(const int32_t *sizes, int p, int n0, int N_lo, int N_hi, int f, uint16_t *x,
                              int64_t capacity, int64_t *offsets, int32_t *status, void *stream) {
    using namespace oob_inst;
    if (!args_ok(p, N_lo, N_hi, f) || !offsets || !status || (!sizes && n0 < 1)) return OOB_EINVAL;
    if (capacity < 0 || (capacity > 0 && !x)) return OOB_EINVAL;
    if (table_bytes(p, N_hi, f) > OOB_INST_STATIC_BYTES) return OOB_ECAPACITY;
    void *ws = nullptr;
    const int rs = static_table(&ws);
    if (rs != OOB_OK) return rs;
    Spec s;
    const int rc = check_spec(sizes, p, n0, N_lo, N_hi, f, ws, OOB_INST_STATIC_BYTES, offsets, status, &s);
    if (rc != OOB_OK) return rc;
    // every entry of the table that is read is written by the counting kernel first: nothing of the
    // previous call's contents survives into this one, and nothing has to be cleared
    const int rl = launch_count(s, offsets, status, (hipStream_t)stream);
    if (rl != OOB_OK) return rl;
    return launch_unrank(s, offsets, status, x, capacity, (hipStream_t)stream);
}

} // extern "C"
