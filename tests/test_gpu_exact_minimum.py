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
    big = dataclasses.replace(inp, fwd_ns=inp.fwd_ns + (1 << 57))  # (N_b + 2) * 8 * 2^57 >= 2^61
    st, _ = P.ExactMinimum(big).run()
    assert st == P.OOB_EOVERFLOW
    ok = dataclasses.replace(inp, fwd_ns=inp.fwd_ns + (1 << 50))
    st, got = P.ExactMinimum(ok).run()
    assert st == P.OOB_OK and got == E.exact_minimum(ok)
