/*
 * oob_dist.h -- C ABI of the batch distribution and plan choice on one gfx950 GPU.
 *
 * Section 4.2.2: a plan (x_j pipelines of template j, one count vector of the instantiation
 * enumeration) distributes the Q = B / b microbatches of an iteration over its pipelines so that
 * the pipelines finish as evenly as possible (Eq. 6: minimise sum_i (N_i T_i - mean)^2 over the
 * pipelines i, N_i microbatches for pipeline i, T_i its time per microbatch), and the plan with
 * the highest throughput is chosen.  The paper calls a general integer solver; here every plan
 * is solved exactly, one plan per GPU lane.
 *
 * Readings (the paper leaves them open): the unknowns are per pipeline and sum to Q; N_i >= 1
 * (a plan with more pipelines than microbatches cannot be distributed); pipelines of one template
 * have the same T, and an optimum gives them counts that differ by at most one, so a distribution
 * is reported per template as (base, extra): `extra` of the template's pipelines take base + 1
 * microbatches, the others base; the throughput of a plan is B over the time of its slowest
 * pipeline, max_i N_i T_i, and of plans with the same time the first in list order is chosen.
 * The minimum of Eq. 6 is unique, the distribution that reaches it need not be: the library
 * reports one.
 *
 * Conventions: as in oob_plan.h -- plain C; array pointers are DEVICE pointers owned by the
 * caller; work is enqueued on `stream`; no call synchronises, copies to or from the host or
 * allocates.  Host-visible argument errors are return codes (OOB_E* of oob_plan.h).
 */
#ifndef OOB_DIST_H
#define OOB_DIST_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define OOB_DIST_MAX_TEMPLATES 1023       /* templates p                                   */
#define OOB_DIST_MAX_TEMPLATES_IN_PLAN 16 /* templates with x_j > 0 in one plan            */
#define OOB_DIST_MAX_Q 65535             /* microbatches per iteration                     */
#define OOB_DIST_MAX_T ((int64_t)1 << 35) /* time per microbatch (about 34 s in ns): keeps every product below 2^127 */

/* Per-plan status. */
#define OOB_DIST_OK 0
#define OOB_DIST_TOO_FEW_MICROBATCHES 1 /* Q < number of pipelines: not distributable        */
#define OOB_DIST_TOO_MANY_TEMPLATES 2   /* more than OOB_DIST_MAX_TEMPLATES_IN_PLAN in use   */
#define OOB_DIST_BAD_TIME 3             /* a template in use has T outside 1..OOB_DIST_MAX_T */
#define OOB_DIST_NO_PIPELINE 4          /* all counts are zero                               */

/* Solves Eq. 6 for `count` plans.
 *   x           [p][capacity] uint16: x[j * capacity + i] = pipelines of template j in plan i
 *               (the layout oob_inst_enumerate writes), capacity >= count
 *   template_T  [p] time per microbatch of a pipeline of template j, p <= OOB_DIST_MAX_TEMPLATES
 *   Q           microbatches per iteration, 1..OOB_DIST_MAX_Q
 *   vx          [count][2] out: x * sum_i (N_i T_i - mean)^2 = x sum a_i^2 - (sum a_i)^2 at the
 *               optimum (x = pipelines of the plan, a_i = N_i T_i), a 128-bit integer as
 *               (low, high) 64-bit words; the minimum of Eq. 6 times x^2, exactly
 *   slowest     [count] out: max_i N_i T_i under the distribution reported
 *   base, extra [p][capacity] uint16 out, or both NULL: the distribution (see above); entries of
 *               templates not in the plan are 0
 *   status      [count] out: OOB_DIST_*; where it is not OOB_DIST_OK the other outputs of the plan
 *               are 0
 * Returns OOB_OK once enqueued, OOB_EINVAL for arguments the host can reject. */
int oob_dist_solve(const uint16_t *x, int64_t count, int64_t capacity, int p, const int64_t *template_T,
                   int Q, uint64_t *vx, int64_t *slowest, uint16_t *base, uint16_t *extra,
                   int32_t *status, void *stream);

/* Chooses, for each of `segments` consecutive groups of plans (offsets[g] .. offsets[g+1]-1, the
 * offsets array of oob_inst_count: one group per cluster size N'), the plan with the smallest
 * `slowest` among those with status OOB_DIST_OK, the first of equals.
 *   count  number of plans the groups cover at most (offsets[segments] - offsets[0] <= count; the
 *          count given to oob_dist_solve): sizes the launch, the groups themselves are read on
 *          the device; plans beyond offsets[segments] are ignored
 *   best   [segments] out: index of the chosen plan, -1 if the group has none
 * Requires oob_dist_solve earlier on the same stream (or completed). */
int oob_dist_choose(const int64_t *offsets, int segments, int64_t count, const int64_t *slowest,
                    const int32_t *status, int64_t *best, void *stream);

#ifdef __cplusplus
}
#endif
#endif
