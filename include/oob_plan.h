/*
 * oob_plan.h -- C ABI of the MI355X pipeline-template planner.
 *
 * The library evaluates, on one gfx950 GPU, the pipeline-template planning
 * dynamic program of the Oobleck paper (Section 4.1): for every node count n
 * of a template range it finds the stage count, the contiguous partition of
 * the model's L layers into stages and the GPUs given to each stage that the
 * paper's divide-and-conquer recursion (Section 4.1.2, Eq. 1-4) selects under
 * the 1F1B iteration-time cost T1 + T2 + T3, and it reports which consecutive
 * template sizes cover every cluster size left after up to f failures
 * (Section 4.1.1 and Appendix A).
 *
 * Conventions
 *   - plain C, no torch types; every array pointer below is a DEVICE pointer
 *     unless it says HOST; the caller owns all of them;
 *   - times are int64 nanoseconds, memory is int64 bytes;
 *   - all work is enqueued on the given HIP stream; the calls do not
 *     synchronise, copy to or from the host, or allocate device memory;
 *   - return value: OOB_OK or a negative OOB_E* code (argument errors, which
 *     the host can see).  Errors that depend on the profile's values are
 *     reported in oob_templates.status on the device;
 *   - one handle must not be used by two calls at the same time (the tables
 *     live in its workspace);
 *   - exact range: inside the tables every time is an exact integer held in a
 *     double.  A profile is accepted (status OOB_OK) iff
 *         (N_b + 4 Smax + 4) * w < 2^52,
 *     where Smax = oob_plan_max_stages(...), N_b = microbatches (4 Smax when
 *     microbatches = 0) and w = sum over the GPU counts d = 1..M of (sum over the
 *     layers of F_{l,d} + B_{l,d}, forbidden entries left out) + sum of all
 *     boundary_ns: a bound on the sum of the stage times of any pipeline that is
 *     loose by about the factor 1 + 1/2 + ... + 1/M.  Otherwise the status is
 *     OOB_EOVERFLOW and nothing else is valid.  The headline workload (98 layers
 *     of about 0.14 s, 8 GPUs per node, N_b = 128) uses 2^44 of the 2^52;
 *   - supported pattern: a handle is created once and used for many calls.
 *     Creating and destroying handles at a high rate is legal (their streams and
 *     events are recycled through a pool of the library) but it is the
 *     one-handle pattern that the tests cover at length.
 */
#ifndef OOB_PLAN_H
#define OOB_PLAN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define OOB_OK 0
#define OOB_EINVAL (-1)    /* bad argument, or (status) a negative time / byte count     */
#define OOB_ECAPACITY (-2) /* exceeds the handle's create-time maxima or its workspace   */
#define OOB_EOVERFLOW (-3) /* (status) costs could reach 2^52 ns: not exactly computable */
#define OOB_EHIP (-4)      /* a HIP runtime call failed                                  */

/* A profile entry >= OOB_FORBIDDEN means "this layer may not run on this many GPUs". */
#define OOB_FORBIDDEN ((int64_t)1 << 62)

#define OOB_MAX_L 1023     /* layers                      */
#define OOB_MAX_NODES 1023 /* nodes of the largest template */
#define OOB_MAX_GPUS 64    /* GPUs per node               */

typedef struct oob_plan oob_plan; /* opaque */

/* Layer profile (Eq. 4, Section 4.1.2: F_{l,d}, B_{l,d}).  DEVICE arrays. */
typedef struct {
    const int64_t *fwd_ns;      /* [L*M]  fwd_ns[l*M + (d-1)] = F_{l,d}, d = 1..M GPUs of one node */
    const int64_t *bwd_ns;      /* [L*M]  B_{l,d}                                                   */
    const int64_t *mem_bytes;   /* [L]    bytes layer l needs in total (model state + activations
                                          of one microbatch); d GPUs each hold ceil(sum / d)        */
    const int64_t *boundary_ns; /* [L]    ns added to a stage whose last layer is l, unless it is
                                          the model's last stage (boundary_ns[L-1] is ignored)      */
} oob_profile;

/* Result buffers.  DEVICE arrays, count = n_max - n_min + 1 templates, template i is for
 * n = n_min + i nodes; Smax = oob_plan_max_stages(...).  A template (Section 3.1, 4.1) is a
 * stage count, the first layer of every stage and the GPUs of every stage. */
typedef struct {
    int32_t *feasible;       /* [count]   1 if a pipeline exists for n nodes under mem_cap          */
    int32_t *S;              /* [count]   stage count ("Choosing the number of stages")            */
    int32_t *kstar;          /* [count]   index of the slowest stage, 0-based (Eq. 2)               */
    int64_t *T;              /* [count]   T1 + T2 + T3, ns                                          */
    int64_t *T1;             /* [count]   Eq. 1                                                     */
    int64_t *T2;             /* [count]   Eq. 2                                                     */
    int64_t *T3;             /* [count]   Eq. 3                                                     */
    int64_t *tmax;           /* [count]   F+B of the slowest stage                                  */
    int32_t *stage_off;      /* [count+1] stage_gpus of template i starts at stage_off[i];
                                          stage_begin of template i starts at stage_off[i] + i      */
    int32_t *stage_begin;    /* [count*(Smax+1)] per template S+1 layer indices, last one = L       */
    int32_t *stage_gpus;     /* [count*Smax]     per template S GPU counts, in node order           */
    int32_t *cover_hdr;      /* [8] n0, n_hi, p, N, (p > n0-1), lo, covered_theorem, covered_tail:
                                    n0 = smallest feasible n, sizes n0..n_hi = the consecutive
                                    feasible counts, N = n_hi + f*n0 (Section 4.1.1);
                                    lo = min((f+1) n0, max(1, N-f));
                                    covered_theorem: every N' in [(f+1) n0, N] is a sum of template
                                    sizes with >= f+1 pipelines (Appendix A);
                                    covered_tail: every N' in [max(1, N-f), N] is such a sum       */
    int32_t *cover_maxpipes; /* [max(count, f+1)] entry N'-lo: largest pipeline count whose sizes
                                    sum to N' (0 = no such sum), N' = lo..N                         */
    int32_t *status;         /* [1] OOB_OK, OOB_EINVAL or OOB_EOVERFLOW; other outputs are
                                    meaningless unless OOB_OK                                       */
    /* HOST fields, written before the call returns (pure functions of the shape) */
    int64_t states;          /* valid (S', u, v, device set) states of the dynamic program         */
    int64_t candidates;      /* (s, k, m) splits examined over all states                           */
} oob_templates;

/* Largest stage count any state can have: min(L, n_max*M, N_b) (N_b = 0: no limit). */
int oob_plan_max_stages(int L, int n_max, int gpus_per_node, int microbatches);

/* Bytes of device workspace a handle for these maxima needs. */
size_t oob_plan_workspace_size(int max_L, int max_nodes, int max_gpus_per_node);

/* Creates a handle over caller-owned device memory (256-byte aligned, at least
 * oob_plan_workspace_size bytes, alive until destroy).  No device memory is allocated.
 * A workspace of k times that size (each share rounded up to 256 bytes; k <= 8) gives the handle
 * k lanes: oob_plan_templates_batch then keeps up to k jobs in flight side by side. */
int oob_plan_create(oob_plan **h, int max_L, int max_nodes, int max_gpus_per_node,
                    void *dev_workspace, size_t workspace_bytes);

/* Plans every template n in [n_min, n_max] (Section 4.1) and the coverage of Section 4.1.1.
 *   L             profile entries (layers)
 *   gpus_per_node M
 *   microbatches  N_b of Eq. 2, used at every level; 0 selects the paper's planning-time
 *                 choice N_b = 4 S' per state
 *   mem_cap       bytes per GPU
 *   f             fault-tolerance threshold
 *   stream        hipStream_t (NULL = default stream)
 * Enqueues, per stage-count level, the split kernel (once or twice: the inner splits of consecutive
 * levels run on two streams of the library beside `stream`, see OOB_OPT_ONE_STREAM) and the select
 * kernel, plus one launch before level 1 (set-up), level 1, and three after the last level
 * (stage counts, stages, coverage). */
int oob_plan_templates(oob_plan *h, const oob_profile *profile, int L, int n_min, int n_max,
                       int gpus_per_node, int microbatches, int64_t mem_cap, int f,
                       oob_templates *out, void *stream);

/* Independent planning jobs.  With one lane (see oob_plan_create) they run one after the other
 * on `stream`; with k lanes job i runs in lane i mod k, the lanes side by side on streams of the
 * library that start after the work already enqueued on `stream` and that `stream` waits for
 * before the call returns, so that the call still looks like work on `stream` to the caller.
 * Every job needs output arrays of its own.
 * All arrays are HOST arrays of length count (of structs / ints holding the per-job values).
 * Returns the first error; jobs before it stay enqueued. */
int oob_plan_templates_batch(oob_plan *h, int count, const oob_profile *profiles, const int *L,
                             const int *n_min, const int *n_max, const int *gpus_per_node,
                             const int *microbatches, const int64_t *mem_cap, const int *f,
                             oob_templates *outs, void *stream);

/* Releases the handle.  The caller must have waited for every call that used it (the streams and
 * events the handle borrowed go back to a pool of the library for the next handle). */
int oob_plan_destroy(oob_plan *h);

/* Launch options of a handle (tests and measurements; every setting gives bit-identical results).
 * Takes effect from the next oob_plan_templates / oob_plan_templates_batch call on.
 *   OOB_OPT_PLAIN_SPLIT  1: the levels S' >= 2 run the tiled split kernel without (total, k) keys,
 *                        which otherwise only serves shapes beyond the keyed kernel's LDS classes
 *                        (hundreds of nodes); default 0
 *   OOB_OPT_XCD_ORDER    1: the workgroup tasks of a level are ordered block row by block row and
 *                        every XCD walks one contiguous stretch of that list (fewer bytes from
 *                        HBM, slightly more time on the headline workload); default 0
 *   OOB_OPT_ONE_STREAM   1: all levels on the caller's stream (no other stream, no events);
 *                        default 0: the inner splits of consecutive levels run on two streams of the
 *                        library beside the caller's, which carries the outer splits and the selects
 *   OOB_OPT_SELECT8_FROM value = first level S' whose select kernel works with eight lanes per
 *                        state (below it: one lane per state); default 82 (the top levels, where
 *                        the select kernel's own latency is what a level waits for)
 *   OOB_OPT_FUSE_FROM    value = first level S' whose two outer splits (s = 1 and s = S'-1) are
 *                        evaluated inside that select kernel instead of by split launches of
 *                        their own; default 82.  A value of 2 covers every level, one above the
 *                        stage limit none
 * Returns OOB_EINVAL for an unknown option. */
#define OOB_OPT_PLAIN_SPLIT 1
#define OOB_OPT_XCD_ORDER 2
#define OOB_OPT_ONE_STREAM 3
#define OOB_OPT_SELECT8_FROM 4
#define OOB_OPT_FUSE_FROM 5
int oob_plan_set_option(oob_plan *h, int option, int value);

/* Test hook, host only (no GPU is touched): checks the table layout and the per-level task lists the
 * library would use for L layers -- every state in exactly one block of its level and at a record of
 * its own, the split-point segments of a block a partition of its range, all counts within the
 * bounds that size a workspace.  Returns 0, a positive number naming the first check that failed,
 * or OOB_EINVAL for L outside 1..OOB_MAX_L. */
int oob_plan_layout_selftest(int L);

/* Measurement hook.  After oob_plan_level_timing(h, 1) every oob_plan_templates call records
 * two HIP events of the handle on its stream, one before the first and one after the last
 * launch of the levels S' >= 2 (the divide/combine step, Eq. 1-3).  oob_plan_last_level_ms
 * waits for the last call's second event and returns the milliseconds between the two, so
 * that the share of the level kernels can be timed without a profiler.  enable = 0 releases
 * the events. */
int oob_plan_level_timing(oob_plan *h, int enable);
int oob_plan_last_level_ms(oob_plan *h, float *ms /* HOST */);

/* Measurement hook: runs a short microbenchmark (independent chains of 32-bit add, compare,
 * select in every lane of every compute unit) on `stream`, waits for it, and returns the
 * measured rate in lane-operations per second: the machine's own figure for the vector-ALU roof
 * that the level kernels are priced against. */
int oob_plan_valu_peak(oob_plan *h, void *stream, double *lane_ops_per_s /* HOST */);

/* The same with the fp64 instruction mix of one candidate of Eq. 1-3 as the split kernels execute it
 * (two adds, a compare, a 64-bit select, a min against a running minimum; eight candidates per
 * step): the rate at which the machine issues that mix when nothing else is in the way. */
int oob_plan_valu_peak_f64(oob_plan *h, void *stream, double *lane_ops_per_s /* HOST */);

/* Introspection for tests: copies the records of (S', delta) left in the workspace by the last
 * oob_plan_templates call into dense DEVICE arrays of n*n entries, n = L - S' + 1, record
 * (u, v) at index u*n + (v - S') (v - u >= S'; other entries read as "no such state").
 * T is the record's total under its own S' (+inf: the state does not exist); choice packs the
 * winning split as s | k << 10 | m << 21.  Device set index: delta = g-1 for g GPUs inside a
 * node (g < M), delta = M-2+a for a whole nodes.  Returns OOB_EINVAL when (S', delta) has no
 * states.  Enqueued on `stream`. */
int oob_plan_export_block(oob_plan *h, int S, int delta, double *T, double *T1, double *tmax,
                          double *T3, int32_t *kstar, int32_t *choice, void *stream);

/* Introspection for tests: copies four int32 flags of the last call to a DEVICE array.
 * flags[0] = 1 when every (total, split point) pair fitted one double key, so that the keyed
 * split kernel did the levels S' >= 2; 0 when the plain split kernel did (totals near the top
 * of the exact range).  Both give identical results.  flags[1..3] are reserved. */
int oob_plan_export_flags(oob_plan *h, int32_t *flags, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* OOB_PLAN_H */
