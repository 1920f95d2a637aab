/*
 * oob_inst.h -- C ABI of the pipeline-instantiation enumeration on one gfx950 GPU.
 *
 * Given the template sizes n_0 < n_1 < ... < n_{p-1} (nodes per pipeline template, Section
 * 4.1.1) the library lists, for every cluster size N' of a range, ALL count vectors
 * (x_0, ..., x_{p-1}) with
 *     x_0 n_0 + ... + x_{p-1} n_{p-1} = N'        (every node is used)
 *     x_0 + ... + x_{p-1} >= f + 1                (at least f+1 pipelines)
 * in the order in which the dynamic program of Section 4.2.1, Eq. 5 lists them:
 *     X(p', N') = X(p'-1, N')  ++  theta(X(p', N' - n_{p'-1}), p'-1)
 * (p' = number of sizes in play; theta adds one to x_{p'-1} of every vector of its list), i.e.
 * ascending with the LAST count compared first.  The second requirement is applied as an
 * order-preserving filter, as in the paper.
 *
 * Conventions: as in oob_plan.h -- plain C; array pointers are DEVICE pointers owned by the
 * caller; work is enqueued on `stream`; no call synchronises, copies to or from the host or
 * allocates.  Host-visible argument errors are return codes (OOB_E* of oob_plan.h); errors that
 * depend on device data are written to *status.
 */
#ifndef OOB_INST_H
#define OOB_INST_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define OOB_INST_MAX_P 1023 /* template sizes            */
#define OOB_INST_MAX_N 4095 /* largest cluster size N'   */
#define OOB_INST_MAX_F 254  /* fault-tolerance threshold */

/* Bytes of device workspace (256-byte aligned) the two calls below need: the table of list
 * lengths |X(p', N')| restricted to "at least q more pipelines", q = 0..f+1
 * ((N_hi+1) (f+2) rows of p+1 64-bit counts, rows padded to a multiple of 8, and a 32-bit
 * copy used while every count is below 2^32).  0 if an argument is out of range. */
size_t oob_inst_workspace_size(int p, int N_hi, int f);

/* First call: list lengths (Eq. 5 with every list replaced by its length).
 *   sizes     [p] template sizes, strictly increasing, >= 1; NULL selects the consecutive
 *             sizes n0, n0+1, ..., n0+p-1 of the node specification (Section 4.1.1)
 *   N_lo..N_hi cluster sizes N' to enumerate (0 <= N_lo <= N_hi <= OOB_INST_MAX_N)
 *   offsets   [N_hi-N_lo+2] out: offsets[i] = number of feasible vectors of all N' < N_lo+i
 *             (exclusive prefix sum); the last entry is the total
 *   status    [1] out: OOB_OK; OOB_EINVAL (sizes not positive and strictly increasing);
 *             OOB_EOVERFLOW (a list is longer than 2^62)
 * Fills the workspace with the table.  One workgroup; the work is p (N_hi+1) (f+2) table
 * entries of at most N_hi / n terms each. */
int oob_inst_count(const int32_t *sizes, int p, int n0, int N_lo, int N_hi, int f,
                   void *dev_workspace, size_t workspace_bytes,
                   int64_t *offsets, int32_t *status, void *stream);

/* Second call: the vectors themselves.  Requires oob_inst_count with the SAME sizes, p, n0,
 * N_lo, N_hi, f, workspace, offsets and status earlier on the same stream (or completed), and
 * the workspace and offsets untouched since: the caller reads offsets' last entry in between to
 * size x.  Structure-of-arrays: vector i of the concatenated lists (N' = N_lo first;
 * offsets[] tells where each N' starts) has its counts at
 *     x[j * capacity + i],  j = 0..p-1                     (uint16: x_j <= N_hi)
 * so that the count of one template over consecutive vectors is contiguous.  Every vector is
 * produced independently from its position in the list.  Does nothing unless *status is
 * OOB_OK; if the total exceeds `capacity` nothing is written and *status = OOB_ECAPACITY.
 * Entries i >= total are left untouched. */
int oob_inst_enumerate(const int32_t *sizes, int p, int n0, int N_lo, int N_hi, int f,
                       void *dev_workspace, size_t workspace_bytes,
                       uint16_t *x, int64_t capacity, const int64_t *offsets, int32_t *status,
                       void *stream);

/* For callers that cannot allocate device memory -- code under HIP graph capture, tight serving
 * loops, harnesses that forbid it: oob_inst_count followed by oob_inst_enumerate as ONE call that
 * takes no workspace.  The count table lives in an array of OOB_INST_STATIC_BYTES bytes that is
 * part of the library's code object: every GPU the library runs on holds it from the first use
 * until the process ends, and no hipMalloc, hipFree or other allocating routine is called.
 *   sizes, p, n0, N_lo, N_hi, f, x, capacity, status, stream   as for the two calls above
 *   offsets   [N_hi-N_lo+2] OUT (written by this call, read by its second kernel)
 * Returns OOB_ECAPACITY, and enqueues nothing, when oob_inst_workspace_size(p, N_hi, f) exceeds
 * OOB_INST_STATIC_BYTES (the headline node specification, 57 sizes up to 128 nodes with f = 8, needs
 * 1 MB); OOB_EINVAL / OOB_EHIP as above.  *status as for oob_inst_enumerate: OOB_ECAPACITY when the
 * total exceeds `capacity` (offsets are still valid, x is untouched), else the vectors are in x.
 * The first call on a GPU looks the array's address up (make it outside a graph capture).  All
 * calls on one GPU share the one array: calls that overlap in time on the same GPU (different
 * streams, or another thread) race and must be serialised by the caller; results of a completed
 * call do not depend on what earlier calls left in the array. */
#define OOB_INST_STATIC_BYTES (4u << 20)
int oob_inst_enumerate_static(const int32_t *sizes, int p, int n0, int N_lo, int N_hi, int f,
                              uint16_t *x, int64_t capacity, int64_t *offsets, int32_t *status,
                              void *stream);

/* Test hook (process-wide): on != 0 makes oob_inst_count keep the table in 64 bits even when every
 * count is below 2^32, so that the path for longer lists can be exercised on cases small enough
 * to enumerate.  Results are identical either way.  Returns the previous setting. */
int oob_inst_keep_wide_table(int on);

#ifdef __cplusplus
}
#endif
#endif /* OOB_INST_H */
