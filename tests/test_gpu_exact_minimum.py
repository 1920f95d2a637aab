"""Exact minimum of the pipeline cost (all explicit pipelines; Section 4.1.2's closed form) through
the C ABI against the CPU oracle: integers, compared exactly."""
import json
import os

import pytest

import inputs
from oracle import exact_minimum as E

pytestmark = pytest.mark.gpu
GOLD = os.path.join(os.path.dirname(__file__), "golden")


@pytest.fixture(scope="module")
def P():
    import torch
    import paper_2309_08125_amd as pkg

    assert torch.cuda.is_available()
    pkg.load()
    return pkg


SHAPES = [(1, 1, 1, 1, 4), (5, 1, 1, 3, 6), (6, 2, 1, 3, 8), (7, 2, 1, 2, 9), (6, 4, 1, 2, 12), (8, 4, 2, 2, 12),
          (9, 2, 2, 3, 9), (12, 3, 1, 4, 12), (15, 2, 1, 5, 15), (23, 8, 1, 3, 30), (37, 3, 1, 5, 40), (20, 16, 1, 2, 33),
          # more GPU positions than one tile of the kernel holds: several blocks of whole nodes
          (12, 8, 1, 10, 12), (10, 4, 2, 20, 10), (14, 3, 1, 30, 14), (9, 16, 1, 6, 9), (30, 5, 1, 27, 30)]


@pytest.mark.parametrize("shape", SHAPES)
def test_small_random_against_the_oracle(P, shape):
    L, M, n_min, n_max, nb = shape
    for seed in range(3):
        for var in ("plain", "tight", "forbid"):
            inp = inputs.random_small(seed, L, M, n_min, n_max, nb, f=1, tight_mem=(var == "tight"),
                                      forbid_some_d=(var == "forbid"))
            print("case", inp.name, shape, var, flush=True)
            st, got = P.ExactMinimum(inp).run()
            assert st == P.OOB_OK and got == E.exact_minimum(inp), (shape, seed, var)


def test_stage_times_that_are_not_monotone_in_the_last_layer(P):
    """A stage that ends at the model's last layer pays no boundary term, so it can be faster than
    the stage ending one layer earlier: the hand case of the oracle's pins (32, 20, 20), and small
    times against boundary terms up to 5 on two hundred seeds."""
    from test_oracle_exact_minimum import boundary_heavy_case

    inp = boundary_heavy_case()
    st, got = P.ExactMinimum(inp).run()
    assert st == P.OOB_OK and got == [32, 20, 20] == E.exact_minimum(inp)
    for seed in range(1000, 1200):
        inp = inputs.random_small(seed, 6, 2, 1, 3, 8, t_lo=1, t_hi=4)
        st, got = P.ExactMinimum(inp).run()
        assert st == P.OOB_OK and got == E.exact_minimum(inp), seed
    for seed in range(40):  # longer models, more GPUs per node
        inp = inputs.random_small(2000 + seed, 14, 4, 1, 4, 16, t_lo=1, t_hi=3)
        st, got = P.ExactMinimum(inp).run()
        assert st == P.OOB_OK and got == E.exact_minimum(inp), seed


MODE_SHAPES = [(7, 3, 1, 2, 0), (6, 2, 1, 3, 0), (8, 1, 1, 4, 0), (12, 4, 1, 3, 0), (25, 8, 1, 4, 0), (40, 2, 1, 9, 0),
               (7, 1, 1, 4, 3), (7, 2, 1, 3, 4), (8, 2, 1, 3, 3), (6, 4, 1, 2, 3), (14, 4, 1, 4, 6), (20, 2, 2, 6, 7),
               (9, 3, 1, 2, 2), (16, 8, 1, 2, 5)]


@pytest.mark.parametrize("shape", MODE_SHAPES)
def test_4S_mode_and_stage_limit_against_the_oracle(P, shape):
    """N_b = 4 S per pipeline (microbatches = 0) and N_b below min(L, n M), where the limit S <= N_b
    binds: the entry point with the stage count in its tables against the oracle that carries it too;
    the one without it against the oracle without it on the templates it answers for, -2 on the others."""
    L, M, n_min, n_max, nb = shape
    for seed in range(3):
        for var in ("plain", "tight", "forbid"):
            inp = inputs.random_small(seed, L, M, n_min, n_max, nb, f=1, tight_mem=(var == "tight"),
                                      forbid_some_d=(var == "forbid"))
            print("case", inp.name, shape, var, flush=True)
            st, got = P.ExactMinimum(inp, staged=True).run()
            assert st == P.OOB_OK and got == E.exact_minimum_staged(inp), (shape, seed, var)
            st, got = P.ExactMinimum(inp).run()
            want = E.exact_minimum(inp, allow_bound=True)  # marks the other templates as the boundary does
            assert E.LIMIT_CAN_BIND == P.OOB_EXACT_LIMIT_CAN_BIND
            assert st == P.OOB_OK and got == want, (shape, seed, var)


def test_stage_limit_at_middle_sizes(P):
    """Tables of 49 x 65 x 21 and 65 x 65 x 33 entries per workgroup, many workgroups in flight."""
    for shape in [(24, 4, 1, 6, 10), (36, 2, 2, 12, 14), (48, 8, 1, 8, 20), (64, 4, 1, 16, 32)]:
        L, M, n_min, n_max, nb = shape
        inp = inputs.random_small(1, L, M, n_min, n_max, nb, f=1)
        print("case", shape, flush=True)
        st, got = P.ExactMinimum(inp, staged=True).run()
        assert st == P.OOB_OK and got == E.exact_minimum_staged(inp), shape


def test_shapes_beyond_lds_take_the_general_path(P):
    """More layers or GPUs per node than the LDS tables hold: the recurrence over tables in the
    workspace, same results."""
    for shape in [(200, 2, 1, 2, 200), (120, 48, 1, 1, 0), (140, 1, 1, 3, 140), (150, 2, 1, 2, 0)]:
        L, M, n_min, n_max, nb = shape
        inp = inputs.random_small(7, L, M, n_min, n_max, nb, f=1, tight_mem=True)
        print("case", shape, flush=True)
        if shape[0] >= 200 or shape[1] >= 48:
            assert P.oob_exact_workspace_size(L, n_max, M) > (16 << 20)   # tables of the workgroups in flight
        st, got = P.ExactMinimum(inp).run()
        assert st == P.OOB_OK and got == E.exact_minimum(inp), shape


@pytest.mark.parametrize("cfg", [1, 2, 3])
def test_configurations_1_to_3(P, cfg):
    inp = inputs.config(cfg)
    st, got = P.ExactMinimum(inp).run()
    assert st == P.OOB_OK and got == E.exact_minimum(inp)
    # never above what the recursion finds
    planner = P.Planner(inp.L, inp.n_max, inp.gpus_per_node)
    res = planner.plan(inp)
    planner.close()
    for i, e in enumerate(got):
        assert (e is None) == (not res["feasible"][i])
        assert e is None or e <= int(res["T"][i])


@pytest.mark.timeout(600)
def test_headline_configuration_against_stored_oracle_results(P):
    """Configuration 4 as bench.py runs it; the oracle's minima are stored by
    tests/golden/make_golden.py cfg4_exact (which calls only the oracle)."""
    inp = inputs.config(4)
    want = json.load(open(os.path.join(GOLD, "cfg4_exact_minimum.json")))["exact_minimum"]
    st, got = P.ExactMinimum(inp).run()
    assert st == P.OOB_OK and got == want
    planner = P.Planner(inp.L, inp.n_max, inp.gpus_per_node)
    res = planner.plan(inp)
    planner.close()
    gaps = [int(res["T"][i]) / e - 1 for i, e in enumerate(got)]
    assert min(gaps) >= 0
    print(f"configuration 4: recursion above the exact minimum by at most {max(gaps):.4%}, "
          f"equal for {sum(g == 0 for g in gaps)} of {len(gaps)} templates", flush=True)


def test_status_for_negative_profile_entries(P):
    import dataclasses

    inp = inputs.random_small(3, 8, 2, 1, 3, 8)
    fwd = inp.fwd_ns.copy()
    fwd[2, 0] = -5
    st, _ = P.ExactMinimum(dataclasses.replace(inp, fwd_ns=fwd)).run()
    assert st == P.OOB_EINVAL
    # several workgroups' worth of (layer, GPU count) pairs, the bad entry in the last one
    inp = inputs.random_small(3, 40, 4, 1, 3, 40)
    fwd = inp.fwd_ns.copy()
    fwd[39, 3] = -1
    st, _ = P.ExactMinimum(dataclasses.replace(inp, fwd_ns=fwd)).run()
    assert st == P.OOB_EINVAL


def test_status_for_times_too_large_to_be_exact(P):
    import dataclasses

    inp = inputs.random_small(4, 8, 2, 1, 3, 8)
    # tables in LDS hold doubles: (N_b + 2) * sum of the layers' slowest times must stay below 2^52
    big = dataclasses.replace(inp, fwd_ns=inp.fwd_ns + (1 << 50))
    st, _ = P.ExactMinimum(big).run()
    assert st == P.OOB_EOVERFLOW
    ok = dataclasses.replace(inp, fwd_ns=inp.fwd_ns + (1 << 44))
    st, got = P.ExactMinimum(ok).run()
    assert st == P.OOB_OK and got == E.exact_minimum(ok)
    # tables in the workspace hold int64: below 2^61
    st, got = P.ExactMinimum(big, staged=True).run()
    assert st == P.OOB_OK and got == E.exact_minimum_staged(big)
    huge = dataclasses.replace(inp, fwd_ns=inp.fwd_ns + (1 << 57))
    st, _ = P.ExactMinimum(huge, staged=True).run()
    assert st == P.OOB_EOVERFLOW


def test_many_random_shapes(P):
    """400 seeded random shapes (1..16 GPUs per node, all three N_b regimes, tight memory, forbidden GPU
    counts, small times against boundary terms) against the oracle; templates whose stage limit can bind
    carry the marker on both sides."""
    import random

    rng = random.Random(2309)
    for n in range(400):
        M = rng.choice([1, 2, 3, 4, 5, 7, 8, 8, 9, 12, 16])
        L = rng.randint(1, 44 if M <= 8 else 30)
        n_max = rng.randint(1, max(1, min(10, L)))
        n_min = rng.randint(1, n_max)
        nb = rng.choice([0, 0, rng.randint(1, 2 * L + 2), L * M + 5, rng.randint(1, 12)])
        var = rng.choice(["plain", "tight", "forbid"])
        kw = {}
        if rng.random() < 0.3:
            kw = dict(t_lo=1, t_hi=rng.choice([3, 4, 8]))
        if rng.random() < 0.2:
            kw["uniform_layers"] = True
        inp = inputs.random_small(rng.randint(0, 10 ** 6), L, M, n_min, n_max, nb, f=1, tight_mem=(var == "tight"),
                                  forbid_some_d=(var == "forbid"), **kw)
        st, got = P.ExactMinimum(inp).run()
        assert st == P.OOB_OK and got == E.exact_minimum(inp, allow_bound=True), (n, L, M, n_min, n_max, nb, var, kw)
