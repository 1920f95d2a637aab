/*
 * oob_exact.h -- C ABI of the exact minimum of the pipeline cost on one gfx950 GPU.
 *
 * The divide-and-conquer recursion of Section 4.1.2 (Eq. 1-3) keeps one record per sub-problem and
 * is therefore a heuristic for the cost it minimises.  This entry point computes the true minimum
 * of that cost (the closed form of Eq. 1-4: sum t + (N_b - S + k* - 1) t_max + sum_{k >= k*} t,
 * k* the first slowest stage) over ALL explicit pipelines of each template: every stage count,
 * every contiguous partition of the layers, every assignment of GPUs in which the stages fill
 * node after node exactly.  The difference to oob_plan_templates' T is the recursion's
 * optimality gap.  Stage time, memory rule and boundary term as in oob_plan.h.
 *
 * Method: with tau the time of the slowest stage the cost is
 *     sum_{i < k*} t_i  +  N_b tau  +  sum_{i > k*} (2 t_i - tau),
 * so for every stage that can be the slowest one, two dynamic programs over (layer, GPUs used)
 * -- before it with stage times < tau, after it with stage times <= tau -- give the best
 * pipeline around it.  The stage-count limit S <= N_b is not modelled: N_b >= min(L, n_max M)
 * is required.
 *
 * Conventions: as in oob_plan.h (DEVICE pointers, caller-owned, enqueued on `stream`, no
 * synchronisation, no allocation; host-visible argument errors are return codes).
 */
#ifndef OOB_EXACT_H
#define OOB_EXACT_H

#include <stddef.h>
#include <stdint.h>

#include "oob_plan.h"

#ifdef __cplusplus
extern "C" {
#endif

#define OOB_EXACT_MAX_L 255      /* layers                                     */
#define OOB_EXACT_MAX_GPUS 4096  /* n_max * gpus_per_node                      */

/* Bytes of device workspace (256-byte aligned): the table of stage times and, for each of the
 * workgroups in flight, the two tables of the dynamic programs.  0 if out of range. */
size_t oob_exact_workspace_size(int L, int n_max, int gpus_per_node);

/*   profile       as for oob_plan_templates (device arrays)
 *   best          [n_max - n_min + 1] out: the exact minimum for n nodes, -1 if no pipeline exists
 *   status        [1] out: OOB_OK; OOB_EINVAL for a negative profile entry; OOB_EOVERFLOW when
 *                 (N_b + 2) w >= 2^61, w = sum over the layers of (largest allowed F + B of the
 *                 layer over the GPU counts) + boundary_ns: every cost stays below (N_b + 2) w, so
 *                 below that bound all int64 arithmetic is exact.  `best` is meaningless unless OOB_OK.
 * Returns OOB_OK once enqueued; OOB_EINVAL for arguments the host can reject, among them
 * microbatches < min(L, n_max * gpus_per_node); OOB_ECAPACITY for a workspace that is too small. */
int oob_exact_minimum(const oob_profile *profile, int L, int n_min, int n_max, int gpus_per_node,
                      int microbatches, int64_t mem_cap, void *dev_workspace, size_t workspace_bytes,
                      int64_t *best, int32_t *status, void *stream);

#ifdef __cplusplus
}
#endif
#endif
