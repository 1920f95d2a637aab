"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests touches the GPU.  Each pins a different part of
oracle/oob_oracle.c to something other than itself: hand-worked values, closed
forms, an exhaustive enumeration, a second evaluation order, invariants.
"""
import json
import os

import numpy as np
import pytest

import inputs
from oracle import brute_force as bf
from oracle import capi
from oracle.topdown import TopDown
from conftest import simple_input

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def stage_times(inp, begins, gpus):
    return [bf.stage_time(inp, begins[i], begins[i + 1], gpus[i]) for i in range(len(gpus))]


# --------------------------------------------------------------------------
# values worked by hand from Eq. 1-4
# --------------------------------------------------------------------------
def test_hand_example_two_stages():
    g = json.load(open(os.path.join(GOLD, "hand_example.json")))
    inp = simple_input(g["fb"], M=g["M"], n_min=g["n"], n_max=g["n"], nb=g["microbatches"])
    # the three cuts, through the closed form
    for k, want in g["cut_costs"].items():
        k = int(k)
        times = [sum(g["fb"][:k]), sum(g["fb"][k:])]
        assert bf.pipeline_cost(times, g["microbatches"])[0] == want
    r = capi.plan(inp)
    t = g["template"]
    assert r["feasible"].tolist() == [1]
    for key in ("S", "T", "T1", "T2", "T3", "kstar", "tmax"):
        assert int(r[key][0]) == t[key], key
    begins, gpus = capi.template_stages(r, 0)
    assert begins == t["stage_begin"] and gpus == t["stage_gpus"]


@pytest.mark.parametrize("nb", [4, 0])
def test_base_case_eq4(nb):
    """Eq. 4: one stage, N_b = 4: T1 = F+B, T2 = 2 (F+B), T3 = F+B.  N_b = 0 is
    the planning-time choice N_b = 4 S', which is 4 at S' = 1."""
    fb = [5, 7, 11]
    inp = simple_input(fb, M=1, n_min=1, n_max=1, nb=nb)
    r = capi.plan(inp)
    t = sum(fb)
    assert (int(r["S"][0]), int(r["T1"][0]), int(r["T2"][0]), int(r["T3"][0])) == (1, t, 2 * t, t)
    assert int(r["T"][0]) == 4 * t and int(r["kstar"][0]) == 0


@pytest.mark.parametrize("L,n,nb,fb", [(8, 2, 8, 5), (12, 4, 16, 3), (12, 3, 6, 7), (6, 6, 12, 2),
                                       (10, 5, 20, 9)])
def test_equal_stages_textbook(L, n, nb, fb):
    """Uniform layers, one GPU per node, n | L: the balanced cut is optimal and
    the 1F1B iteration time is the textbook (N_b + S - 1) * stage time."""
    inp = simple_input([fb] * L, M=1, n_min=n, n_max=n, nb=nb)
    r = capi.plan(inp)
    assert int(r["S"][0]) == n
    assert int(r["T"][0]) == (nb + n - 1) * (L // n) * fb
    begins, gpus = capi.template_stages(r, 0)
    assert begins == [i * (L // n) for i in range(n + 1)]


def test_slowest_stage_tie_goes_left():
    """Two equal stages: k* = 0, so T2 = (N_b - 2 - 1) t, T3 = 2 t."""
    inp = simple_input([4, 4], M=1, n_min=2, n_max=2, nb=10)
    r = capi.plan(inp)
    assert int(r["kstar"][0]) == 0
    assert (int(r["T1"][0]), int(r["T2"][0]), int(r["T3"][0])) == (8, 7 * 4, 8)


def test_slowest_stage_on_the_right():
    """Stage times [2, 6]: k* = 1, T2 = (N_b - 2 + 1 - 1) 6, T3 = 6 (Eq. 2-3)."""
    inp = simple_input([2, 6], M=1, n_min=2, n_max=2, nb=10)
    r = capi.plan(inp)
    assert int(r["kstar"][0]) == 1
    assert (int(r["T1"][0]), int(r["T2"][0]), int(r["T3"][0])) == (8, 8 * 6, 6)


def test_candidate_tie_break_smallest_k():
    """[2,1,1,2] on two nodes: cuts k=1,2,3 give stage times [2,4],[3,3],[4,2].
    N_b=3: costs 6+(3-2+1-1)*4+4=14, 6+0*3+6=12, 6+0*4+6=12 -> k=2 wins the tie
    with k=3."""
    inp = simple_input([2, 1, 1, 2], M=1, n_min=2, n_max=2, nb=3)
    r = capi.plan(inp)
    assert int(r["T"][0]) == 12
    assert capi.template_stages(r, 0)[0] == [0, 2, 4]


def test_boundary_term_charged_to_non_last_stages():
    inp = simple_input([3, 3], M=1, n_min=2, n_max=2, nb=4, bnd=[10, 99])
    r = capi.plan(inp)
    # stage times [13, 3]; the last layer's boundary time is ignored
    assert (int(r["T1"][0]), int(r["tmax"][0]), int(r["kstar"][0])) == (16, 13, 0)
    assert int(r["T"][0]) == 16 + (4 - 2 - 1) * 13 + 16


def test_memory_cap_forces_more_gpus():
    """ceil(bytes / d) <= cap decides feasibility per stage."""
    inp = simple_input([8, 8], M=2, n_min=1, n_max=1, nb=4, mem=[5, 5], cap=5)
    r = capi.plan(inp)
    # one stage on both GPUs holds ceil(10/2) = 5 <= 5: feasible; two stages of 1 GPU: 5 each
    assert r["feasible"].tolist() == [1]
    inp = simple_input([8, 8], M=2, n_min=1, n_max=1, nb=4, mem=[5, 6], cap=5)
    r = capi.plan(inp)
    assert r["feasible"].tolist() == [0]  # 11 bytes: ceil(11/2)=6 > 5, and a 6-byte layer alone > 5
    assert r["cover_hdr"].tolist() == [0] * 8


def test_forbidden_gpu_count():
    fbd = [[4, 1 << 62], [4, 2]]
    inp = simple_input([4, 4], M=2, n_min=1, n_max=1, nb=4, fb_by_d=fbd)
    r = capi.plan(inp)
    # layer 0 may not run on 2 GPUs -> single stage on 2 GPUs impossible; two stages of 1 GPU each
    assert int(r["S"][0]) == 2 and capi.template_stages(r, 0)[1] == [1, 1]


# --------------------------------------------------------------------------
# closed form, invariants, second evaluation order, exhaustive enumeration
# --------------------------------------------------------------------------
def check_invariants(inp, r):
    L, M = inp.L, inp.gpus_per_node
    for i in range(inp.n_max - inp.n_min + 1):
        n = inp.n_min + i
        if not r["feasible"][i]:
            continue
        S = int(r["S"][i])
        begins, gpus = capi.template_stages(r, i)
        hi = min(L, n * M, inp.microbatches if inp.microbatches > 0 else L)
        assert n <= S <= hi
        assert begins[0] == 0 and begins[-1] == L
        assert all(b1 > b0 for b0, b1 in zip(begins, begins[1:]))
        assert sum(gpus) == n * M
        acc = 0  # stages pack the nodes in order without straddling
        for gcount in gpus:
            assert 1 <= gcount <= M
            acc += gcount
            assert acc <= M
            if acc == M:
                acc = 0
        assert acc == 0
        times = stage_times(inp, begins, gpus)
        assert all(t is not None for t in times)  # memory cap and forbidden d respected
        nb = inp.microbatches if inp.microbatches > 0 else 4 * S
        T, T1, T2, T3, kstar = bf.pipeline_cost(times, nb)
        got = tuple(int(r[k][i]) for k in ("T", "T1", "T2", "T3", "kstar", "tmax"))
        assert got == (T, T1, T2, T3, kstar, max(times))


SMALL = [
    # L, M, n_min, n_max, nb
    (5, 1, 1, 3, 6), (6, 2, 1, 3, 8), (7, 2, 1, 2, 5), (6, 4, 1, 2, 12), (8, 4, 2, 2, 12),
    (6, 3, 1, 2, 0), (7, 1, 1, 4, 0), (5, 2, 1, 2, 3),
]


@pytest.mark.parametrize("shape", SMALL)
@pytest.mark.parametrize("variant", ["plain", "tight", "forbid"])
def test_against_topdown_and_brute_force(shape, variant):
    L, M, n_min, n_max, nb = shape
    never_below, equal = 0, 0
    for seed in range(6):
        inp = inputs.random_small(seed, L, M, n_min, n_max, nb, f=1,
                                  tight_mem=(variant == "tight"),
                                  forbid_some_d=(variant == "forbid"))
        r = capi.plan(inp)
        check_invariants(inp, r)
        td = TopDown(inp)
        for i in range(n_max - n_min + 1):
            n = n_min + i
            t = td.template(n)
            b = bf.brute_min(inp, n)
            assert (t is None) == (not r["feasible"][i])
            if t is None:
                # the recursion reaches every packing, so it fails only if no pipeline exists
                assert b is None
                continue
            begins, gpus = capi.template_stages(r, i)
            assert [(u, v, g) for (u, v), g in zip(zip(begins, begins[1:]), gpus)] == t["stages"]
            for key in ("T", "S", "T1", "T3", "tmax", "kstar"):
                assert int(r[key][i]) == t[key], (key, seed, n)
            assert b is not None and int(r["T"][i]) >= b[0]
            never_below += 1
            equal += int(r["T"][i]) == b[0]
    # The recursion keeps one record per sub-problem, chosen under the sub-problem's own
    # stage count, so it is a heuristic: equality with the exhaustive minimum is a
    # statistic (most instances), never a rule.
    assert never_below > 0 and equal * 2 >= never_below, (equal, never_below)
    print(f"shape {shape} {variant}: recursion == exhaustive minimum in {equal}/{never_below}")


def test_exhaustive_when_every_split_joins_single_stages():
    """With at most two stages every candidate is a pair of base cases, so the
    recursion is an exhaustive search and must equal the brute-force minimum."""
    for seed in range(40):
        for (L, M, n) in [(6, 1, 2), (6, 2, 1), (7, 1, 2)]:
            inp = inputs.random_small(seed, L, M, n, n, nb=7, tight_mem=(seed % 2 == 0))
            r = capi.plan(inp)
            b = bf.brute_min(inp, n)
            if b is None:
                assert not r["feasible"][0]
            else:
                assert int(r["T"][0]) == b[0]


def test_state_tables_match_topdown_everywhere():
    """Every state the recursion visits, all fields, against the bottom-up tables."""
    for seed, (L, M, n_max, nb) in enumerate([(7, 3, 3, 9), (8, 2, 3, 0), (6, 4, 2, 5)]):
        inp = inputs.random_small(100 + seed, L, M, 1, n_max, nb, tight_mem=(seed == 0))
        o = capi.Oracle(inp)
        td = TopDown(inp)
        for n in range(1, n_max + 1):
            td.template(n)
        checked = 0
        for (S, u, v, dev), rec in td.memo.items():
            delta = dev[1] - 1 if dev[0] == "G" else M - 2 + dev[1]
            if not td.possible(S, dev) or v - u < S:
                continue
            blk = o.block(S, delta)
            assert bool(blk["exists"][u, v]) == (rec is not None)
            if rec is not None:
                assert (int(blk["T1"][u, v]), int(blk["T3"][u, v]), int(blk["tmax"][u, v]),
                        int(blk["kstar"][u, v])) == rec[:4]
                if S > 1:
                    assert (int(blk["s"][u, v]), int(blk["k"][u, v]), int(blk["m"][u, v])) == rec[4]
                assert int(blk["T"][u, v]) == td.total(S, rec)
                checked += 1
        assert checked > 50
        o.close()


# --------------------------------------------------------------------------
# metamorphic properties
# --------------------------------------------------------------------------
def test_scaling_times_scales_costs():
    inp = inputs.random_small(5, 9, 2, 1, 3, 10)
    r1 = capi.plan(inp)
    c = 7
    inp2 = inputs.PlanInput("x", inp.fwd_ns * c, inp.bwd_ns * c, inp.mem_bytes, inp.boundary_ns * c,
                            inp.n_min, inp.n_max, inp.gpus_per_node, inp.microbatches, inp.mem_cap,
                            inp.f)
    r2 = capi.plan(inp2)
    for k in ("T", "T1", "T2", "T3", "tmax"):
        assert (r2[k] == c * r1[k]).all()
    for k in ("S", "kstar", "stage_begin", "stage_gpus", "feasible"):
        assert (r2[k] == r1[k]).all()


def test_memo_property_larger_range_keeps_smaller_templates():
    """Section 4.1.2, memoisation: the tables of the largest template contain the
    smaller ones, so asking for more node counts changes nothing below."""
    inp = inputs.random_small(9, 9, 2, 1, 2, 12)
    big = inputs.random_small(9, 9, 2, 1, 4, 12)
    r1, r2 = capi.plan(inp), capi.plan(big)
    for k in ("feasible", "S", "T", "T1", "T2", "T3", "kstar", "tmax"):
        assert (r1[k] == r2[k][:2]).all()
    for i in range(2):
        assert capi.template_stages(r1, i) == capi.template_stages(r2, i)


def test_raising_cap_never_raises_a_cost():
    for seed in range(10):
        a = inputs.random_small(seed, 7, 2, 1, 2, 9, tight_mem=True)
        b = inputs.PlanInput("x", a.fwd_ns, a.bwd_ns, a.mem_bytes, a.boundary_ns, a.n_min, a.n_max,
                             a.gpus_per_node, a.microbatches, a.mem_cap + 3, a.f)
        ra, rb = capi.plan(a), capi.plan(b)
        for i in range(2):
            if ra["feasible"][i]:
                assert rb["feasible"][i]
                # feasibility is monotone in the cap for the recursion (it reaches every
                # packing); cost monotonicity is only guaranteed for the exhaustive minimum
                bmin_a, bmin_b = bf.brute_min(a, 1 + i), bf.brute_min(b, 1 + i)
                assert bmin_b[0] <= bmin_a[0]


# --------------------------------------------------------------------------
# structural work counts (pure functions of L, M, n_max, N_b)
# --------------------------------------------------------------------------
def test_work_counts_config1_by_hand():
    """M = 1 forces S' = a.  States: intervals of length >= a for a = 1..4 over 12
    layers = 78 + 66 + 55 + 45 = 244.  Candidates: s = m, one per inner cut:
    sum_len (13-len)(len-1) = 286 for a=2, 2*220 for a=3, 3*165 for a=4 -> 1221."""
    r = capi.plan(inputs.config(1))
    assert (r["states"], r["candidates"]) == (244, 1221)


def test_work_counts_configs_2_3():
    assert capi.plan(inputs.config(2))["states"] == 21035
    r3 = capi.plan(inputs.config(3))
    assert r3["states"] == 76226 and 1.51e7 < r3["candidates"] < 1.53e7


def test_configs_1_to_3_invariants():
    for c in (1, 2, 3):
        inp = inputs.config(c)
        r = capi.plan(inp)
        assert r["feasible"].all()
        check_invariants(inp, r)


def test_stored_digests_of_the_batched_configuration_are_the_oracles():
    """tests/golden/cfg5_all_templates.json (written by make_golden.py cfg5_all, which calls only the
    oracle) is what the GPU path is compared with at full size: the three shortest instances are
    recomputed here and must reproduce their stored digest and their stored T, S and feasibility."""
    import hashlib
    import json
    import os

    import parity_util as PU

    path = os.path.join(os.path.dirname(__file__), "golden", "cfg5_all_templates.json")
    stored = json.load(open(path))["instances"]
    insts = inputs.config(5)
    for idx in sorted((int(k) for k in stored), key=lambda k: insts[k].L)[:3]:
        inp, want = insts[idx], stored[str(idx)]
        cnt = inp.n_max - inp.n_min + 1
        t = capi.plan(inp)
        assert [int(x) for x in t["T"][:cnt]] == want["T"] and [int(x) for x in t["S"][:cnt]] == want["S"]
        assert [int(x) for x in t["feasible"][:cnt]] == want["feasible"]
        assert hashlib.sha256(PU.canonical_templates(t, cnt, inp.f)).hexdigest() == want["sha256"]
