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
 *     sum_{i < k*} t_i  +  N_b tau  +  sum_{i > k*} (2 t_i - tau)                       (N_b given)
 *     sum_{i < k*} (t_i + 4 tau)  +  4 tau  +  sum_{i > k*} (2 t_i + 3 tau)             (N_b = 4 S)
 * so for every stage that can be the slowest one, two dynamic programs -- before it with stage
 * times < tau, after it with stage times <= tau -- give the best pipeline around it.
 *
 * Two entry points.  oob_exact_minimum keeps no stage count in its tables: it answers for the
 * templates whose stage-count limit S <= N_b cannot bind (microbatches = 0, the paper's planning-time
 * choice N_b = 4 S per pipeline, or microbatches >= min(L, n gpus_per_node)) and reports -2 for
 * the others.  oob_exact_minimum_staged carries the stage count as a third table index and answers
 * for every template and every N_b; its tables live in the workspace and its work grows with the
 * stage limit: for small and middle sizes.
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

/* Bytes of device workspace (256-byte aligned) of oob_exact_minimum: three tables of stage times
 * (the dynamic programs themselves run in LDS); for shapes whose tables exceed LDS also the tables
 * of the workgroups in flight.  0 if out of range. */
size_t oob_exact_workspace_size(int L, int n_max, int gpus_per_node);

/* Bytes of device workspace of oob_exact_minimum_staged: the stage-time tables and about a gigabyte
 * of tables (at least 16 workgroups' worth; the entry point uses as many as the workspace it is
 * given holds, at least 16).  0 if out of range. */
size_t oob_exact_staged_workspace_size(int L, int n_max, int gpus_per_node, int microbatches);

/*   profile       as for oob_plan_templates (device arrays)
 *   microbatches  N_b; 0 selects N_b = 4 S per pipeline
 *   best          [n_max - n_min + 1] out: the exact minimum for n nodes; -1 if no pipeline exists;
 *                 -2 (oob_exact_minimum only) if the limit S <= N_b can bind for this template
 *   status        [1] out: OOB_OK; OOB_EINVAL for a negative profile entry; OOB_EOVERFLOW when
 *                 mult w reaches the exact range, w = sum over the layers of (largest allowed F + B
 *                 of the layer over the GPU counts) + boundary_ns, mult = N_b + 2 (4 min(L, n_max
 *                 gpus_per_node) + 2 for N_b = 4 S): every cost stays below mult w.  The range is
 *                 2^52 where the tables are held in LDS as doubles (oob_exact_minimum on shapes up to
 *                 about 128 layers and 16 GPUs per node), 2^61 otherwise.  `best` is meaningless
 *                 unless OOB_OK.
 * Return OOB_OK once enqueued; OOB_EINVAL for arguments the host can reject; OOB_ECAPACITY for a
 * workspace that is too small. */
int oob_exact_minimum(const oob_profile *profile, int L, int n_min, int n_max, int gpus_per_node,
                      int microbatches, int64_t mem_cap, void *dev_workspace, size_t workspace_bytes,
                      int64_t *best, int32_t *status, void *stream);
int oob_exact_minimum_staged(const oob_profile *profile, int L, int n_min, int n_max, int gpus_per_node,
                             int microbatches, int64_t mem_cap, void *dev_workspace, size_t workspace_bytes,
                             int64_t *best, int32_t *status, void *stream);

#ifdef __cplusplus
}
#endif
#endif
