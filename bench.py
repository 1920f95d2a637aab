#!/usr/bin/env python3
"""Benchmark of the template-planning hot path on one MI355X.

A step = one whole oob_plan_templates call (set-up, level 1, every level S' >= 2, template
extraction, coverage) on the GPT-175B-shaped workload (98 profile entries, templates for
8..64 nodes x 8 GPUs, 128 microbatches) with the profile already resident in HBM.
Prints ONE JSON line.  Metric: dynamic-program states per second (structural count of valid
states, 3 724 666 per step for the headline workload) and wall-ms per full template set.
The same line carries, as objects of their own and outside the timed steps, the later stages
on the node specification the planner produced: `instantiation` (Section 4.2.1), `distribution`
(Section 4.2.2) and `reconfiguration` (Section 5.1), each with its own roofline.
`--config 5` times the batch of 256 independent jobs instead.
"""
import argparse
import dataclasses
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# Arithmetic per candidate split (s, k, m) as the level kernels execute it (Eq. 1-3 with the child's
# own total stored, every time an exact integer in a double): 2 adds, 1 compare, 2 selects, 1 min
# = 6 fp64 vector instructions.  gfx950 issues fp64 add / min / compare / select at one lane
# per SIMD lane and clock: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz = 39.3 T lane-instructions/s
# (half of the 78.6 TFLOP/s quoted for fp64 FMA, which counts two flops per lane-instruction).
# `roofline.frac` = structural candidates x 6 / time of the level launches / that peak.
FP64_OPS_PER_CANDIDATE = 6
PEAK_LANE_OPS = 256 * 64 * 2.4e9
# The same work in the int64 formulation of Eq. 1-3 (4 adds, one 64-bit compare with 3 selects, one
# 64x32 multiply, one (cost, index) compare-and-select: about 30 32-bit lane operations), kept as
# a secondary figure under `int64_formulation` (how the run compares with an int64 kernel at the
# 32-bit integer roof of the same 39.3 T lane-op/s; a ratio, not a roofline fraction).
INT64_OPS_PER_CANDIDATE = 30
# Constants copied from the tracked profile of the level kernels on configuration 4
# (profiles/k_split_key_config4.md; not measured by this script): HBM bytes per call from the two
# rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE over all level kernels, each scaled by what the same
# counter reads for one 256 MiB device-to-device copy), and vector-ALU wave-instructions per call
# (SQ_INSTS_VALU of k_split_key + k_select).
PROFILE_CONFIG4 = {"source": "profiles/k_split_key_config4.md",
                   "hbm_read_bytes_per_call": 19.29e9, "hbm_written_bytes_per_call": 6.27e9,
                   "valu_wave_insts_per_call": 3.06e9 + 0.07e9,
                   "kernel_launches_per_call": 277}  # 175 k_split_key + 97 k_select / k_select8 + 5 others (kernel trace)


def median(xs):
    xs = sorted(xs)
    return xs[len(xs) // 2]


def cpu_baseline(inp):
    """The CPU oracle, as it stands, on a bounded sample of the same workload: all host threads
    on the templates for the smaller half of the node counts, and one thread on the two smallest
    templates; each the median of three runs."""
    from oracle import capi

    cores = capi.lib().oob_oracle_threads()
    sample = dataclasses.replace(inp, n_max=min(inp.n_max, 32 if cores >= 16 else 16))

    def timed(job, threads):
        runs = []
        for _ in range(3):
            t0 = time.time()
            o = capi.Oracle(job, threads=threads)
            runs.append((time.time() - t0, o.states, o.candidates))
            o.close()
        return median(runs), [round(r[0], 2) for r in runs]

    (dt, states, cands), runs = timed(sample, 0)
    res = {"value": states / dt, "unit": "states/s", "cores": cores,
           "kind": "oracle", "seconds": round(dt, 2), "runs_seconds": runs, "candidates_per_s": cands / dt,
           "sample": f"same profile, templates for {sample.n_min}..{sample.n_max} nodes: "
                     f"{states} states, {cands} candidates; median of 3 runs"}
    one = dataclasses.replace(inp, n_max=min(inp.n_max, inp.n_min + 1))
    (dt, states, cands), runs = timed(one, 1)
    res["single_thread"] = {"value": states / dt, "unit": "states/s", "cores": 1, "seconds": round(dt, 2),
                            "runs_seconds": runs, "candidates_per_s": cands / dt,
                            "sample": f"templates for {one.n_min}..{one.n_max} nodes: {states} states, "
                                      f"{cands} candidates; median of 3 runs"}
    return res


def call_latency(P, planner, inp, reps=7):
    """One call at a time, from a profile in host memory to the results in host memory: the four
    profile arrays are copied to the device, oob_plan_templates is enqueued, and the host waits for
    the templates, the stage lists and the coverage to arrive (wall clock around all of it)."""
    import torch

    out = planner.new_outputs(inp)
    times = []
    for _ in range(reps + 1):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        prof = P.DeviceProfile(inp)
        planner.enqueue(prof, out)
        res = out.to_host()
        times.append((time.perf_counter() - t0) * 1e3)
        assert int(res["status"][0]) == 0
    return {"median": median(times[1:]), "min": min(times[1:]), "max": max(times[1:]), "calls": reps,
            "what": "host clock: H2D of the profile (one copy), all kernels of one oob_plan_templates call, D2H of "
                    "every result array (one copy); one call at a time, first call dropped"}


def bench_instantiation(P, inp, res, reps=20):
    """Section 4.2.1 on the node specification the planner just produced: every count vector for
    every N' from (f+1) n0 to N.  Timed with events on the stream the kernels are launched on."""
    import torch

    n0, n_hi, p, N = (int(v) for v in res["cover_hdr"][:4])
    if p < 1:
        return None
    inst = P.Instantiator(None, (inp.f + 1) * n0, N, inp.f, n0=n0, p=p)
    off, st = inst.count()
    total = int(off[-1])
    if st != P.OOB_OK or total == 0:
        return {"status": st, "vectors": total}
    cap = (total + 63) // 64 * 64  # rows of x start on 128-byte lines
    x = torch.empty((p, cap), dtype=torch.int16, device="cuda")
    stream = torch.cuda.current_stream()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    inst.enqueue(x, cap)
    torch.cuda.synchronize()
    ev[0].record(stream)
    for _ in range(reps):
        P.oob_inst_count(*inst._spec(), inst.offsets.data_ptr(), inst.status.data_ptr(), stream.cuda_stream)
    ev[1].record(stream)
    for _ in range(reps):
        inst.enqueue(x, cap)
    ev[2].record(stream)
    torch.cuda.synchronize()
    t_count, t_enum = ev[0].elapsed_time(ev[1]) / reps * 1e-3, ev[1].elapsed_time(ev[2]) / reps * 1e-3
    nbytes = 2.0 * p * total  # algorithmic: every count of every vector written once (uint16)
    return {"workload": f"template sizes {n0}..{n_hi}, f={inp.f}, N'={(inp.f + 1) * n0}..{N}",
            "vectors": total, "templates": p, "count_us": t_count * 1e6, "enumerate_us": t_enum * 1e6,
            "value": total / t_enum, "unit": "count vectors/s",
            "roofline": {"bound": "hbm", "achieved": nbytes / t_enum / 1e9, "peak": 8000.0, "unit": "GB/s",
                         "frac": nbytes / t_enum / 8e12,
                         # rocprofv3 --pmc of this kernel on configuration 4's node specification, scaled as
                         # above: 149 557 KiB written + 694 KiB read per launch (profiles/k_inst_unrank_config4.md)
                         "traffic": (149557 + 694) * 1024 if (n0, n_hi, inp.f) == (8, 64, 8) else None,
                         "kernel": "k_inst_unrank", "bytes_per_vector": 2 * p}}


def exact_relaxations(inp):
    """Relaxations (one stage appended to one partial cover: an add and a min) that the exact-minimum
    kernel evaluates on this job, counted on the host from the stage times alone: for every possible
    slowest stage (u, v, d) with time tau, the one-node tables before u and after v -- a stage on dd
    GPUs into layer p reaches back over the layers whose stage time stays below tau (at most to the
    table's start layer q) and serves M - dd + 1 GPU counts -- plus the node-level recurrences.
    Returns (possible slowest stages, one-node relaxations, node-level relaxations)."""
    import numpy as np

    L, M, n_max = inp.L, inp.gpus_per_node, inp.n_max
    fb = (inp.fwd_ns + inp.bwd_ns).astype(np.float64)
    forb = (inp.fwd_ns >= (1 << 62)) | (inp.bwd_ns >= (1 << 62))
    fb[forb] = 0
    PT = np.vstack([np.zeros((1, M)), np.cumsum(fb, axis=0)])
    PF = np.vstack([np.zeros((1, M)), np.cumsum(forb, axis=0)])
    PM = np.concatenate([[0], np.cumsum(inp.mem_bytes.astype(np.int64))])
    d = np.arange(1, M + 1)
    t0 = np.full((L + 1, L + 1, M), np.inf)  # stage time without the boundary term, inf = impossible
    for u in range(L):
        for v in range(u + 1, L + 1):
            ok = (PF[v] - PF[u] == 0) & (-(-(PM[v] - PM[u]) // d) <= inp.mem_cap)
            t0[u, v, ok] = (PT[v] - PT[u])[ok]
    bnd = np.concatenate([[0], inp.boundary_ns.astype(np.float64)])
    bnd[L] = 0
    t = t0 + bnd[None, :, None]
    uu, vv, dd = np.nonzero(np.isfinite(t))
    taus = t[uu, vv, dd]
    w = (M - d + 1).astype(np.float64)

    def h(cnt, j):  # sum_{i=1..j} min(cnt, i): the table starts q = p-1 .. p-j against a reach of cnt layers
        c = np.minimum(cnt, j)
        return c * (c + 1) / 2 + c * (j - c)

    pre_rows = np.zeros((len(taus), L + 1))
    suf_rows = np.zeros((len(taus), L + 1))
    for p in range(1, L + 1):
        for k in range(M):
            pre_rows[:, p] += w[k] * h(np.searchsorted(t[p - 1::-1, p, k], taus, side="left"), p)
    for p in range(L):
        for k in range(M):
            suf_rows[:, p] += w[k] * h(np.searchsorted(t0[p, p + 1:, k], taus, side="right"), L - p)
    pre = np.cumsum(pre_rows, axis=1)[np.arange(len(taus)), uu]
    suf = np.cumsum(suf_rows[:, ::-1], axis=1)[:, ::-1][np.arange(len(taus)), vv]
    lu, lv = uu.astype(np.float64), (L - vv).astype(np.float64)
    node = (np.minimum(n_max, lu + 1) * (lu * (lu + 1) / 2 + (M - 1) * lu) +
            np.minimum(n_max, lv + 1) * (lv * (lv + 1) / 2 + (M - 1) * lv))
    return len(taus), float(pre.sum() + suf.sum()), float(node.sum())


def bench_exact(P, planner, inp, res, reps=3):
    """The exact minimum of the template cost for every template of the workload, under the workload's
    N_b and under N_b = 4 S (the paper's planning-time choice), and the gap of the recursion's result
    to each.  Timed with events on the stream the kernels are launched on; the oracle (all host cores)
    is timed on the same job when that takes seconds, else on a part of it."""
    import torch
    from oracle import capi, exact_minimum

    out = {}
    stream = torch.cuda.current_stream()
    for mode, job, plan in (("given_nb", inp, res),
                            ("nb_4S", dataclasses.replace(inp, microbatches=0), None)):
        if plan is None:
            plan = planner.plan(job)
        ex = P.ExactMinimum(job)
        st, got = ex.run()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        ev[0].record(stream)
        for _ in range(reps):
            ex.enqueue()
        ev[1].record(stream)
        torch.cuda.synchronize()
        dt = ev[0].elapsed_time(ev[1]) / reps * 1e-3
        assert st == P.OOB_OK, "exact minimum"
        answered = [(i, e) for i, e in enumerate(got) if e is not None and e != P.OOB_EXACT_LIMIT_CAN_BIND]
        gaps = [int(plan["T"][i]) / e - 1 for i, e in answered]
        assert all(g >= 0 for g in gaps), "the recursion below the exact minimum"
        out[mode] = {"ms": dt * 1e3, "templates_answered": len(answered), "templates": len(got),
                     "recursion_gap_max": max(gaps) if gaps else None,
                     "recursion_exact_for": sum(g == 0 for g in gaps)}
        if mode == "given_nb":
            got_given, dt_given = got, dt
    small = dataclasses.replace(inp, n_max=min(inp.n_max, inp.n_min + 7)) if capi.lib().oob_oracle_threads() < 16 else inp
    t0 = time.time()
    want = exact_minimum.exact_minimum(small, allow_bound=True)
    t_cpu = time.time() - t0
    tight = [exact_minimum.is_tight(small, n) for n in range(small.n_min, small.n_max + 1)]
    assert [w for w, ok in zip(want, tight) if ok] == [g for g, ok in zip(got_given, tight) if ok], \
        "exact minimum against the oracle"
    ncand, relax_node_tables, relax_node_level = exact_relaxations(inp)
    relax = relax_node_tables + relax_node_level
    ops = 2  # per relaxation: one fp64 add and one fp64 min
    out.update({
        "workload": f"{len(got_given)} templates, {ncand} possible slowest stages, {relax:.4g} relaxations "
                    f"({relax_node_tables:.4g} in one-node tables, {relax_node_level:.4g} node-level), counted on the host",
        "ms": dt_given * 1e3, "value": len(got_given) / dt_given, "unit": "templates/s",
        "roofline": {"bound": "alu", "achieved": relax * ops / dt_given / 1e12, "peak": PEAK_LANE_OPS / 1e12,
                     "unit": "T fp64 lane-instr/s", "frac": relax * ops / dt_given / PEAK_LANE_OPS, "traffic": None,
                     "kernel": "k_exact_lds", "ops_per_relaxation": ops, "relaxations_per_s": relax / dt_given,
                     "note": "relaxations actually evaluated (host count); the kernel is bound by LDS and "
                             "dependent-load latency at two waves per SIMD, not by the vector ALUs"},
        "cpu_baseline": {"seconds": t_cpu, "cores": capi.lib().oob_oracle_threads(), "kind": "oracle",
                         "sample": f"templates for {small.n_min}..{small.n_max} nodes, N_b = {inp.microbatches}"}})
    return out


def bench_distribution(P, inp, res, Q=512, reps=3, oracle_sample=40):
    """Section 4.2.2 on every plan the enumeration of this node specification lists: Eq. 6 solved
    exactly per plan (time per microbatch of a template = its T1), then the best plan per cluster
    size.  Timed with events on the stream the kernels are launched on; the oracle on a sample."""
    import numpy as np
    import torch
    from oracle import batch_distribution

    n0, n_hi, p, N = (int(v) for v in res["cover_hdr"][:4])
    if p < 1:
        return None
    tT = [int(v) for v in res["T1"][n0 - inp.n_min: n0 - inp.n_min + p]]
    if max(tT) > (1 << 35) or min(tT) < 1:
        return None
    inst = P.Instantiator(None, (inp.f + 1) * n0, N, inp.f, n0=n0, p=p)
    off, st = inst.count()
    total = int(off[-1])
    if st != P.OOB_OK or total == 0:
        return None
    x = torch.empty((p, total), dtype=torch.int16, device="cuda")
    inst.enqueue(x, total)
    d = P.Distributor(x, total, tT, Q, distribution=True)
    stream = torch.cuda.current_stream()
    d.enqueue()
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    ev[0].record(stream)
    for _ in range(reps):
        d.enqueue()
    ev[1].record(stream)
    torch.cuda.synchronize()
    dt = ev[0].elapsed_time(ev[1]) / reps * 1e-3
    status, vx, slow, base, extra = d.solve()
    best = d.choose(off)
    t_choose = d.time_choose(off)
    assert (status == P.OOB_DIST_OK).all(), "distribution"
    X = x.cpu().numpy().view("uint16").T
    rng = np.random.Generator(np.random.PCG64(1))
    sample = rng.integers(0, total, size=oracle_sample).tolist()
    t0 = time.time()
    for i in sample:
        assert batch_distribution.sweep(batch_distribution.pipelines_of(X[i].tolist(), tT), Q)[0] == vx[i], i
    cpu = oracle_sample / (time.time() - t0)
    # algorithmic HBM bytes per plan: its counts in, base and extra out (2 bytes each per template), 28 bytes of results
    nbytes = total * (6.0 * p + 28)
    return {"workload": f"all {total} plans of template sizes {n0}..{n_hi}, f={inp.f}, N'={(inp.f + 1) * n0}..{N}; "
                        f"{Q} microbatches; time per microbatch = T1 of the template",
            "value": total / dt, "unit": "plans/s", "ms": dt * 1e3, "choose_us": t_choose * 1e6,
            "best_plan_for_all_nodes": X[int(best[-1])].nonzero()[0].tolist() if best[-1] >= 0 else None,
            # bound by instruction issue: 25 119 vector instructions per wave of 64 plans (SQ_INSTS_VALU / SQ_WAVES
            # of profiles/k_dist_solve_config4.md, a constant of that profile, not measured here), each 4 cycles
            # on one of 1024 SIMDs; the algorithmic HBM bytes are kept as a secondary figure
            "roofline": {"bound": "alu", "achieved": total / 64 * 25119 * 64 / dt / 1e12, "peak": PEAK_LANE_OPS / 1e12,
                         "unit": "T lane-instr/s (32/64-bit integer)", "frac": total / 64 * 25119 * 64 / dt / PEAK_LANE_OPS,
                         "traffic": None, "kernel": "k_dist_solve", "valu_insts_per_wave_from_profile": 25119,
                         "hbm_algorithmic": {"bytes_per_plan": 6 * p + 28, "GB_per_s": nbytes / dt / 1e9,
                                             "frac_of_hbm_peak": nbytes / dt / 8e12}},
            "cpu_baseline": {"value": cpu, "unit": "plans/s", "cores": 1, "kind": "oracle",
                             "sample": f"{oracle_sample} of the plans"}}


def bench_reconfiguration(P, inp, res, trajectories=1 << 20, reps=5, oracle_sample=64):
    """Section 5.1 on the node specification the planner just produced: `trajectories` failure
    sequences, one node lost per step, from N nodes down to the end of training.  Timed with events
    on the stream the kernel is launched on; the oracle is timed on a sample of the trajectories."""
    import torch
    import inputs
    from oracle import reconfiguration

    n0, n_hi, p, N = (int(v) for v in res["cover_hdr"][:4])
    if p < 1 or N // n0 > 64:
        return None
    sizes0 = inputs.starting_pipelines(4, n0, n_hi, N, inp.f).tolist()
    steps = N - (inp.f + 1) * n0 + 1
    draws = inputs.failure_draws(4, steps, 1, trajectories)
    sim = P.FailureSimulator(sizes0, n0, n_hi, inp.f, draws)
    stream = torch.cuda.current_stream()
    sim.enqueue()
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    ev[0].record(stream)
    for _ in range(reps):
        sim.enqueue()
    ev[1].record(stream)
    torch.cuda.synchronize()
    dt = ev[0].elapsed_time(ev[1]) / reps * 1e-3
    st, summary, final, trace = sim.run()
    assert st == P.OOB_OK and not summary["violations"].any(), "reconfiguration"
    t0 = time.time()
    for t in range(oracle_sample):
        reconfiguration.simulate(sizes0, n0, n_hi, inp.f, draws[:, :, t])
    cpu = oracle_sample * steps / (time.time() - t0)
    # algorithmic HBM bytes: one draw read and one trace word written per step, summary and final sizes once
    nbytes = trajectories * (8.0 * steps + 4 * (len(sizes0) + 8))
    return {"workload": f"template sizes {n0}..{n_hi}, f={inp.f}, {N} nodes in {len(sizes0)} pipelines, "
                        f"{trajectories} failure sequences of {steps} single-node failures",
            "value": trajectories * steps / dt, "unit": "repaired failures/s", "ms": dt * 1e3,
            "merges_per_sequence": float(summary["merges"].mean()),
            "borrowed_per_sequence": float(summary["borrowed"].mean()),
            "roofline": {"bound": "hbm", "achieved": nbytes / dt / 1e9, "peak": 8000.0, "unit": "GB/s",
                         "frac": nbytes / dt / 8e12, "traffic": None, "kernel": "k_reconf",
                         "bytes_per_step": 8},
            "cpu_baseline": {"value": cpu, "unit": "repaired failures/s", "cores": 1, "kind": "oracle",
                             "sample": f"{oracle_sample} of the sequences"}}


def batch_exact_gaps(P, insts, results, staged_instances=4):
    """Gap of the recursion to the exact minimum over the batched workload.  The kernel without stage
    counts answers for the templates whose limit S <= N_b cannot bind (all templates of the instances
    with L <= N_b, the templates up to N_b / M nodes of the others); the kernel with stage counts, whose
    work grows with the fourth power of L, answers for every template of the few shortest instances
    beyond that."""
    import torch

    t0 = time.time()
    gaps, answered, total = [], 0, 0
    for inp, res in zip(insts, results):
        st, got = P.ExactMinimum(inp).run()
        assert st == P.OOB_OK
        for i, e in enumerate(got):
            total += 1
            if e is not None and e != P.OOB_EXACT_LIMIT_CAN_BIND:
                answered += 1
                gaps.append(int(res["T"][i]) / e - 1)
    t_fast = time.time() - t0
    assert min(gaps) >= 0
    out = {"without_stage_counts": {"instances": len(insts), "templates": total, "templates_answered": answered,
                                    "recursion_gap_max": max(gaps), "recursion_gap_mean": sum(gaps) / len(gaps),
                                    "recursion_exact_for": sum(g == 0 for g in gaps), "seconds": round(t_fast, 2)}}
    order = sorted((k for k, i in enumerate(insts) if i.L > i.microbatches), key=lambda k: insts[k].L)[:staged_instances]
    gaps, t0 = [], time.time()
    for k in order:
        inp = insts[k]
        nbytes = P.oob_exact_staged_workspace_size(inp.L, inp.n_max, inp.gpus_per_node, inp.microbatches)
        st, got = P.ExactMinimum(inp, staged=True, workspace_bytes=8 * nbytes).run()
        assert st == P.OOB_OK
        gaps += [int(results[k]["T"][i]) / e - 1 for i, e in enumerate(got) if e is not None]
        torch.cuda.empty_cache()
    if order:
        assert min(gaps) >= 0
        out["with_stage_counts"] = {"instances": [insts[k].name for k in order], "L": [insts[k].L for k in order],
                                    "templates_answered": len(gaps), "recursion_gap_max": max(gaps),
                                    "recursion_gap_mean": sum(gaps) / len(gaps),
                                    "recursion_exact_for": sum(g == 0 for g in gaps),
                                    "seconds": round(time.time() - t0, 2)}
    return out


def bench_batch(P, insts, args):
    """Configuration 5: 256 independent instances through oob_plan_templates_batch, profiles
    resident in HBM; a step is the whole batch."""
    import torch

    planner = P.Planner(max(i.L for i in insts), max(i.n_max for i in insts), max(i.gpus_per_node for i in insts),
                        lanes=args.lanes)
    profs = [P.DeviceProfile(i) for i in insts]
    outs = [planner.new_outputs(i) for i in insts]
    stream = torch.cuda.current_stream()

    def run():
        rc = P.oob_plan_templates_batch(planner.h, [p.c for p in profs], [i.L for i in insts],
                                        [i.n_min for i in insts], [i.n_max for i in insts],
                                        [i.gpus_per_node for i in insts], [i.microbatches for i in insts],
                                        [i.mem_cap for i in insts], [i.f for i in insts], [o.c for o in outs],
                                        stream.cuda_stream)
        assert rc == P.OOB_OK

    for _ in range(args.warmup):
        run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    assert all(int(o.t["status"].item()) == 0 for o in outs), "device status"
    states = sum(o.c.states for o in outs)
    cands = sum(o.c.candidates for o in outs)
    achieved = cands * FP64_OPS_PER_CANDIDATE * args.steps / elapsed
    exact = batch_exact_gaps(P, insts, [o.to_host() for o in outs]) if not args.no_exact else None
    print(json.dumps({
        "metric": "DP states/sec (wall-ms per batch of 256 instances in ms_per_step)",
        "value": states * args.steps / elapsed, "unit": "states/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": elapsed / args.steps * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f64 (exact integers < 2^52; int64 in and out)",
        "data": "synthetic",
        "config": {"workload": "config 5: 256 instances, L=24..128, templates n=1..32 x 8 GPUs, N_b=64",
                   "lanes": args.lanes,
                   "states": states, "candidates": cands},
        "roofline": {"bound": "alu", "achieved": achieved / 1e12, "peak": PEAK_LANE_OPS / 1e12,
                     "unit": "T fp64 lane-instr/s", "frac": achieved / PEAK_LANE_OPS, "traffic": None,
                     "kernel": "whole batched call (all kernels, host enqueue included)",
                     "ops_per_candidate": FP64_OPS_PER_CANDIDATE},
        "exact_minimum": exact}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=4,
                    help="workload 1-4 (default: headline 4); 5 = the batch of 256 instances (one batched call per step)")
    ap.add_argument("--lanes", type=int, default=4,
                    help="--config 5 only: jobs of the batch in flight side by side (workspace for that many)")
    ap.add_argument("--paper-nb", action="store_true",
                    help="N_b = 4 S' per state (the paper's planning-time choice) instead of the configuration's N_b")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-exact", action="store_true", help="--config 5 only: skip the exact-minimum gaps")
    ap.add_argument("--calibrate-copy-mib", type=int, default=0,
                    help="before the steps, run one device-to-device copy of this many MiB (a plain "
                         "copy kernel of known size, to scale rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build plans on ONE GPU (no collectives); run with --gpus 1. "
              "The '8 GPUs' of the workload are the cluster being planned for.", file=sys.stderr)
        sys.exit(2)

    import torch
    import inputs
    import paper_2309_08125_amd as P

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    from paper_2309_08125_amd import build as hip_build

    hip_build.ensure_built()  # loads what is built; compiles only if there is no library
    if args.config == 5:
        return bench_batch(P, inputs.config(5), args)
    inp = inputs.config(args.config)
    if args.paper_nb:
        inp = dataclasses.replace(inp, microbatches=0, name=inp.name + "_paper_nb")
    planner = P.Planner(inp.L, inp.n_max, inp.gpus_per_node)
    prof = P.DeviceProfile(inp)
    out = planner.new_outputs(inp)
    planner.level_timing(True)

    if args.calibrate_copy_mib > 0:
        src = torch.ones(args.calibrate_copy_mib << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        planner.enqueue(prof, out)
    torch.cuda.synchronize()
    # the timed region: K calls back to back, no synchronisation in between
    t0 = time.perf_counter()
    for _ in range(args.steps):
        planner.enqueue(prof, out)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    # the same K calls again for the roofline: each call's level launches are bracketed by HIP events
    # on the caller's stream, read (with a wait for the second event) after every call
    level_ms = []
    for _ in range(args.steps):
        planner.enqueue(prof, out)
        level_ms.append(planner.last_level_ms())
    torch.cuda.synchronize()

    res = out.to_host()
    assert int(res["status"][0]) == 0, "device status"
    states, cands = res["states"], res["candidates"]
    Smax = P.oob_plan_max_stages(inp.L, inp.n_max, inp.gpus_per_node, inp.microbatches)
    launches = max(1, Smax - 1)
    lvl_ms = sum(level_ms) / len(level_ms)
    achieved = cands * FP64_OPS_PER_CANDIDATE / (lvl_ms * 1e-3)
    measured_peak = planner.valu_peak()  # add / compare / select microbenchmark on this GPU
    measured_peak_f64 = planner.valu_peak(f64_mix=True)  # the fp64 mix of a candidate, alone on the machine
    prof4 = PROFILE_CONFIG4 if args.config == 4 and not args.paper_nb else None
    line = {
        "metric": "DP states/sec (wall-ms per full template set in ms_per_step)",
        "value": states * args.steps / elapsed,
        "unit": "states/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64 (exact integers < 2^52; int64 in and out)",
        "data": "synthetic",
        "config": {"workload": f"config {args.config}: {inp.name}, L={inp.L} profile entries, "
                               f"templates n={inp.n_min}..{inp.n_max} x {inp.gpus_per_node} GPUs, "
                               f"N_b={inp.microbatches if inp.microbatches else '4S (per state)'}, f={inp.f}",
                   "states": states, "candidates": cands, "levels": Smax},
        "latency_ms": call_latency(P, planner, inp),
        "roofline": {"bound": "alu", "achieved": achieved / 1e12, "peak": PEAK_LANE_OPS / 1e12,
                     "unit": "T fp64 lane-instr/s", "frac": achieved / PEAK_LANE_OPS,
                     "traffic": ((prof4["hbm_read_bytes_per_call"] + prof4["hbm_written_bytes_per_call"]) / launches
                                 if prof4 else None),
                     "traffic_unit": "HBM bytes per level (one launch group), rocprofv3 --pmc",
                     "kernel": "level kernels S'>=2 (divide/combine, Eq. 1-3): k_split_key + k_select / k_select8",
                     "ops_per_candidate": FP64_OPS_PER_CANDIDATE, "launches": launches,
                     "avg_launch_ms": lvl_ms / launches, "levels_ms_per_step": lvl_ms,
                     "candidates_per_s": cands / (lvl_ms * 1e-3),
                     "measured_peak_int32": measured_peak / 1e12,
                     "measured_peak_fp64_candidate_mix": measured_peak_f64 / 1e12,
                     "frac_of_measured_fp64_mix": achieved / measured_peak_f64,
                     "int64_formulation": {"ops_per_candidate": INT64_OPS_PER_CANDIDATE,
                                           "lane_ops_per_s": cands * INT64_OPS_PER_CANDIDATE / (lvl_ms * 1e-3) / 1e12,
                                           "ratio_to_int32_peak": cands * INT64_OPS_PER_CANDIDATE / (lvl_ms * 1e-3)
                                                                  / PEAK_LANE_OPS,
                                           "note": "a ratio to an int64 kernel running at the roof, not a "
                                                   "roofline fraction"},
                     "from_profile": ({"source": prof4["source"], "constants_not_measured_in_this_run": True,
                                       "valu_issue_utilisation": prof4["valu_wave_insts_per_call"] * 4
                                                                 / (1024 * 2.4e9 * lvl_ms * 1e-3),
                                       "valu_lane_insts_per_candidate": prof4["valu_wave_insts_per_call"] * 64 / cands,
                                       "kernel_launches_per_call": prof4["kernel_launches_per_call"]}
                                      if prof4 else None)},
    }
    line["instantiation"] = bench_instantiation(P, inp, res)
    line["reconfiguration"] = bench_reconfiguration(P, inp, res)
    line["distribution"] = bench_distribution(P, inp, res)
    line["exact_minimum"] = bench_exact(P, planner, inp, res)
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(inp)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
