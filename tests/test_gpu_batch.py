"""Batched heterogeneous planning (256 independent instances) through the C ABI.

Small and middle instances are compared bit for bit with the CPU oracle run in the test (every
state record of the last one); the largest instance with stored oracle results (every state record,
as digests per level); and all 256, at full size, with the oracle's templates, stage lists and
coverage stored as one digest per instance, plus properties that hold for any correct output
(structural invariants of every template and the closed-form cost of its own stages).
"""
import os
import sys
import time

import numpy as np
import pytest

import inputs
from oracle import brute_force as bf
from oracle import capi
import parity_util as PU
from test_gpu_parity import check_against_golden, full_check, oracle_expected

pytestmark = pytest.mark.gpu
GOLD = os.path.join(os.path.dirname(__file__), "golden")


@pytest.fixture(scope="module")
def P():
    import torch
    import paper_2309_08125_amd as pkg

    assert torch.cuda.is_available()
    pkg.load()
    return pkg


@pytest.fixture(scope="module")
def instances():
    return inputs.config(5)


def check_properties(P, inp, r):
    """Invariants + closed form, for every template of one result."""
    assert int(r["status"][0]) == 0
    L, M = inp.L, inp.gpus_per_node
    for i in range(inp.n_max - inp.n_min + 1):
        n = inp.n_min + i
        if not r["feasible"][i]:
            continue
        S = int(r["S"][i])
        begins, gpus = P.template_stages(r, i)
        assert n <= S <= min(L, n * M, inp.microbatches if inp.microbatches > 0 else L)
        assert begins[0] == 0 and begins[-1] == L and all(b > a for a, b in zip(begins, begins[1:]))
        assert sum(gpus) == n * M
        acc = 0
        for g in gpus:  # stages fill node after node exactly
            assert 1 <= g <= M
            acc += g
            assert acc <= M
            acc %= M
        assert acc == 0
        times = [bf.stage_time(inp, begins[q], begins[q + 1], gpus[q]) for q in range(S)]
        assert all(t is not None for t in times)  # memory cap respected
        nb = inp.microbatches if inp.microbatches > 0 else 4 * S
        T, T1, T2, T3, kstar = bf.pipeline_cost(times, nb)
        got = tuple(int(r[k][i]) for k in ("T", "T1", "T2", "T3", "kstar", "tmax"))
        assert got == (T, T1, T2, T3, kstar, max(times)), (inp.name, n)
    # coverage header is consistent with the feasibility flags
    feas = np.flatnonzero(r["feasible"])
    if len(feas):
        n0 = inp.n_min + int(feas[0])
        assert int(r["cover_hdr"][0]) == n0
        want = capi.coverage(r["feasible"], inp.n_min, inp.f)
        assert np.array_equal(r["cover_hdr"], want["hdr"])
        assert np.array_equal(r["cover_maxpipes"][:len(want["maxpipes"])], want["maxpipes"])


def test_batch_small_and_middle_instances_against_oracle(P, instances):
    """Ragged batch (L = 24 .. 47, f = 2 .. 8) through oob_plan_templates_batch."""
    order = sorted(range(len(instances)), key=lambda i: instances[i].L)
    picks = order[:5] + [i for i in order if 40 <= instances[i].L <= 47][:3]
    batch = [instances[i] for i in picks]
    planner = P.Planner(max(b.L for b in batch), 32, 8)
    results = planner.plan_batch(batch)
    for inp, got in zip(batch, results):
        print(f"instance {inp.name} L={inp.L} f={inp.f}", flush=True)
        o, want = oracle_expected(inp)
        o.close()
        PU.compare_templates(got, want, inp.n_max - inp.n_min + 1)
        check_properties(P, inp, got)
    # every state of the last job of the batch (its tables are the ones left in the workspace)
    full_check(P, planner, batch[-1])
    planner.close()


def test_batch_on_several_lanes_against_oracle(P, instances):
    """A workspace for three jobs: the jobs of a batch run three at a time side by side (job i in
    lane i mod 3).  Ragged batch of eight, every template against the oracle, and every state of
    the last job, whose tables are in lane 1."""
    order = sorted(range(len(instances)), key=lambda i: instances[i].L)
    batch = [instances[i] for i in order[:4] + order[60:62] + order[5:7]]
    planner = P.Planner(max(b.L for b in batch), 32, 8, lanes=3)
    for rep in range(2):  # the second batch reuses the lanes' streams and events
        results = planner.plan_batch(batch)
        for inp, got in zip(batch, results):
            print(f"lanes: instance {inp.name} L={inp.L} f={inp.f}", flush=True)
            o, want = oracle_expected(inp)
            o.close()
            PU.compare_templates(got, want, inp.n_max - inp.n_min + 1)
    for S in (1, 2, 7):  # the last job ran in lane 7 mod 3 = 1: its tables are read from there
        o, _ = oracle_expected(batch[-1])
        for delta in range(o.D):
            gb = planner.block(S, delta)
            assert (gb is not None) == o.valid(S, delta)
            if gb is not None:
                PU.compare_block(gb, o.block(S, delta), S, batch[-1].L)
        o.close()
    # a single call after a batch runs in lane 0 again
    full_check(P, planner, batch[0])
    planner.close()


@pytest.mark.timeout(900)
def test_largest_instance_against_stored_oracle_results(P, instances):
    """L = 128, 32 nodes x 8 GPUs, N_b = 64: 3.5e10 candidates; oracle results stored by
    tests/golden/make_golden.py cfg5 45."""
    inp = instances[45]
    assert inp.L == 128
    got = check_against_golden(P, inp, os.path.join(GOLD, "cfg5_45_expected.json"))
    check_properties(P, inp, got)


@pytest.mark.timeout(900)
def test_all_256_instances_against_stored_oracle_results(P, instances):
    """The whole batched workload at full size: 4.8e8 states, 1.9e12 candidates.  Every instance's
    templates, stage lists, coverage and work counters against the oracle's, stored by
    tests/golden/make_golden.py cfg5_all as one SHA-256 per instance over everything
    parity_util.compare_templates compares (plus feasibility, S and T per template in the clear, so that
    a mismatch names the template)."""
    import hashlib
    import json

    stored = json.load(open(os.path.join(GOLD, "cfg5_all_templates.json")))["instances"]
    assert len(stored) == len(instances) == 256
    planner = P.Planner(128, 32, 8)
    lanes4 = P.Planner(128, 32, 8, lanes=4)  # the same jobs four at a time: identical results
    t0 = time.time()
    states = cands = 0
    for lo in range(0, len(instances), 32):  # 8 calls of 32 jobs keep the result buffers small
        chunk = instances[lo: lo + 32]
        results = planner.plan_batch(chunk)
        for r, r4 in zip(results, lanes4.plan_batch(chunk)):
            assert r.keys() == r4.keys()
            for k in r:
                assert np.array_equal(r[k], r4[k]), k
        for idx, (inp, r) in enumerate(zip(chunk, results), start=lo):
            want = stored[str(idx)]
            cnt = inp.n_max - inp.n_min + 1
            assert (want["name"], want["L"], want["f"]) == (inp.name, inp.L, inp.f)
            assert int(r["status"][0]) == 0
            for k in ("feasible", "S", "T"):
                got = [int(x) for x in r[k][:cnt]]
                assert got == want[k], f"instance {idx} ({inp.name}): {k} differs at template " \
                                       f"{next(i for i in range(cnt) if got[i] != want[k][i])}"
            assert hashlib.sha256(PU.canonical_templates(r, cnt, inp.f)).hexdigest() == want["sha256"], \
                f"instance {idx} ({inp.name}): stage lists, cost terms or coverage differ"
            check_properties(P, inp, r)
            states += r["states"]
            cands += r["candidates"]
        print(f"instances {lo}..{lo + len(chunk) - 1} done, {time.time() - t0:.1f} s", flush=True)
    # structural counts of the whole batch (closed-form sums over the 256 shapes)
    assert (states, cands) == (483151346, 1931782435821)
    print(f"256 instances: {states} states, {cands} candidates in {time.time() - t0:.1f} s "
          f"(GPU planning + comparison with the stored oracle digests + host-side property checks)", flush=True)
    planner.close()
    lanes4.close()
