/*
 * oob_reconf.h -- C ABI of the reconfiguration simulator on one gfx950 GPU.
 *
 * Pipeline reinstantiation after node failures (Section 5.1: simple reinstantiation, borrowing
 * nodes, merging pipelines; Appendix B: a merged pipeline always finds a template), run for many
 * independent failure sequences at once, one trajectory per GPU lane.  The state of a trajectory
 * is the list of running pipelines, each a node count out of the template sizes
 * n0, n0+1, ..., n_hi of the node specification (Section 4.1.1).
 *
 * One step loses `burst` nodes and then repairs every affected pipeline, in list order:
 *   - draw r selects node floor(r * (nodes left) / 2^32), nodes counted pipeline after pipeline in
 *     list order;
 *   - if fewer than (f+1) n0 nodes are left after the losses, training stops for good (Section 5)
 *     and the step repairs nothing;
 *   - a pipeline that still has at least n0 nodes is reinstantiated from the template of its new
 *     size;
 *   - a pipeline below n0 borrows one node at a time from the largest pipeline above n0 (the
 *     first of equals) until it has n0;
 *   - when nobody can lend, it absorbs the smallest other pipeline (the first of equals), again
 *     and again until it has n0; it keeps its list position, the absorbed one leaves the list.
 * Which lender and which partner is this library's reading: the paper leaves both open.
 *
 * Conventions: as in oob_plan.h -- plain C; array pointers are DEVICE pointers owned by the
 * caller; work is enqueued on `stream`; the call neither synchronises nor copies to or from the
 * host nor allocates.  Host-visible argument errors are return codes (OOB_E* of oob_plan.h);
 * errors that depend on device data are written to *status.
 */
#ifndef OOB_RECONF_H
#define OOB_RECONF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define OOB_RECONF_MAX_PIPELINES 64  /* pipelines at the start            */
#define OOB_RECONF_MAX_BURST 255     /* nodes lost per step               */
#define OOB_RECONF_MAX_NODES 65535   /* nodes at the start                */

#define OOB_RECONF_STOP_NONE 0
#define OOB_RECONF_STOP_TOO_FEW_NODES 1 /* fewer than (f+1) n0 nodes left           */
#define OOB_RECONF_STOP_NO_PARTNER 2    /* a short pipeline found nobody to absorb  */

/* Fields of a trace word (one per step and trajectory). */
#define OOB_RECONF_TRACE_REINSTANTIATED(w) ((w) & 0xffu)        /* pipelines repaired by step 1     */
#define OOB_RECONF_TRACE_BORROWED(w) (((w) >> 8) & 0xffu)       /* nodes moved by step 2            */
#define OOB_RECONF_TRACE_MERGES(w) (((w) >> 16) & 0x7fu)        /* pipelines absorbed by step 3     */
#define OOB_RECONF_TRACE_ALIVE(w) (((w) >> 23) & 0x7fu)         /* pipelines after the step         */
#define OOB_RECONF_TRACE_STOP(w) ((w) >> 30)                    /* OOB_RECONF_STOP_* after the step */

/* Rows of `summary` (row k of trajectory t at summary[k * T + t]). */
enum {
    OOB_RECONF_SURVIVED = 0,   /* steps repaired before training stopped                         */
    OOB_RECONF_REINSTANTIATED, /* totals of the three trace counts over the repaired steps ...   */
    OOB_RECONF_BORROWED,
    OOB_RECONF_MERGES,
    OOB_RECONF_ALIVE,          /* pipelines at the end                                           */
    OOB_RECONF_NODES,          /* nodes at the end                                               */
    OOB_RECONF_VIOLATIONS,     /* bit 0: a repaired pipeline ended above n_hi (no template, the  */
                               /* claim of Appendix B failed); bit 1: fewer than f+1 pipelines   */
                               /* after a repair                                                 */
    OOB_RECONF_STOP,           /* OOB_RECONF_STOP_* at the end                                   */
    OOB_RECONF_SUMMARY_ROWS
};

/* Runs T trajectories of `steps` steps from the same starting pipelines.
 *   sizes0       [c0] nodes of each starting pipeline, n0 <= sizes0[i] <= n_hi,
 *                1 <= c0 <= OOB_RECONF_MAX_PIPELINES, sum <= OOB_RECONF_MAX_NODES
 *   n0, n_hi, f  node specification (smallest and largest template, Section 4.1.1) and the
 *                fault-tolerance threshold
 *   draws        [steps][burst][T] 32-bit draws, trajectory index fastest
 *   trace        [steps][T] out, or NULL: one word per step (macros above); steps after the stop
 *                repeat the stop code and the pipeline count with zero counts
 *   final_sizes  [c0][T] out, or NULL: nodes per starting list position at the end, 0 = absorbed
 *   summary      [OOB_RECONF_SUMMARY_ROWS][T] out
 *   status       [1] out: OOB_OK, or OOB_EINVAL when sizes0 is outside [n0, n_hi] or too large in
 *                sum (then nothing else is written)
 * Returns OOB_OK once enqueued, OOB_EINVAL for arguments the host can reject (nothing is
 * enqueued then), OOB_EHIP for a launch error. */
int oob_reconf_simulate(const int32_t *sizes0, int c0, int n0, int n_hi, int f,
                        const uint32_t *draws, int steps, int burst, int64_t T,
                        uint32_t *trace, int32_t *final_sizes, int32_t *summary,
                        int32_t *status, void *stream);

#ifdef __cplusplus
}
#endif
#endif
