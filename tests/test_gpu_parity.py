"""Parity of the HIP path with the CPU oracle, through the C ABI, on a real MI355X.

Integer work: everything must match bit for bit -- every field of every state record of
every level, the templates, the stage lists, the coverage and the work counters.
"""
import hashlib
import json
import os
import sys

import numpy as np
import pytest

import inputs
from oracle import capi
import parity_util as PU

pytestmark = pytest.mark.gpu
GOLD = os.path.join(os.path.dirname(__file__), "golden")


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def P():
    import torch
    import paper_2309_08125_amd as pkg

    assert torch.cuda.is_available(), "GPU tests need a GPU"
    pkg.load()
    return pkg


def oracle_expected(inp):
    o = capi.Oracle(inp)
    want = o.templates(inp.n_min, inp.n_max)
    c = capi.coverage(want["feasible"], inp.n_min, inp.f)
    want["cover_hdr"], want["cover_maxpipes"] = c["hdr"], c["maxpipes"]
    want["states"], want["candidates"] = o.states, o.candidates
    return o, want


def full_check(P, planner, inp):
    """Templates and every block of every level against the oracle."""
    say(f"case {inp.name} L={inp.L} M={inp.gpus_per_node} n={inp.n_min}-{inp.n_max} "
        f"nb={inp.microbatches} f={inp.f} cap={inp.mem_cap}")
    got = planner.plan(inp)
    o, want = oracle_expected(inp)
    try:
        PU.compare_templates(got, want, inp.n_max - inp.n_min + 1)
        nstates = 0
        for S in range(1, o.Smax + 1):
            for delta in range(o.D):
                gb = planner.block(S, delta)
                assert (gb is not None) == o.valid(S, delta), (S, delta)
                if gb is not None:
                    nstates += PU.compare_block(gb, o.block(S, delta), S, inp.L)
        return got, nstates
    finally:
        o.close()


SHAPES = [(5, 1, 1, 3, 6), (6, 2, 1, 3, 8), (7, 2, 1, 2, 5), (6, 4, 1, 2, 12), (8, 4, 2, 3, 12),
          (6, 3, 1, 2, 0), (7, 1, 1, 4, 0), (9, 3, 1, 4, 4), (12, 2, 2, 5, 0), (10, 8, 1, 2, 16),
          (1, 1, 1, 1, 4), (1, 4, 1, 2, 4), (3, 2, 1, 5, 2), (37, 3, 1, 5, 9), (70, 2, 1, 6, 11),
          # more than 64 target device sets (two workgroup groups), 16 GPUs per node, many nodes
          (72, 1, 1, 70, 0), (20, 16, 1, 2, 8), (40, 2, 1, 40, 64), (30, 3, 2, 30, 0),
          # the largest node the library takes: 64 GPUs (OOB_MAX_GPUS), 63 device sets inside it
          (40, 64, 1, 1, 0), (20, 64, 1, 2, 24)]


@pytest.mark.parametrize("shape", SHAPES)
def test_small_random_every_state(P, shape):
    """Small and ragged shapes (L not a multiple of any tile, L = 1, more nodes than layers,
    N_b below the stage limit, the paper's N_b = 4 S' mode), three variants of the memory cap /
    forbidden GPU counts, every state compared."""
    L, M, n_min, n_max, nb = shape
    planner = P.Planner(L, n_max, M)
    for seed in range(3):
        for var in ("plain", "tight", "forbid"):
            inp = inputs.random_small(seed, L, M, n_min, n_max, nb, f=seed,
                                      tight_mem=(var == "tight"), forbid_some_d=(var == "forbid"))
            full_check(P, planner, inp)
    planner.close()


def test_longest_model_the_library_takes(P):
    """OOB_MAX_L layers (1023): 129 x 129 blocks of the plane, up to 128 segments per block."""
    planner = P.Planner(1023, 2, 1)
    full_check(P, planner, inputs.random_small(5, 1023, 1, 1, 2, 0, f=1))
    planner.close()
    planner = P.Planner(300, 2, 2)
    full_check(P, planner, inputs.random_small(5, 300, 2, 1, 2, 5, f=1))
    planner.close()


def test_many_random_shapes_on_one_handle(P):
    """Four hundred random shapes (L, GPUs per node, template range, N_b, f, memory and
    forbidden-GPU-count variants, large times, uniform layers) back to back on one handle, every
    state of every case against the oracle."""
    import random

    rng = random.Random(2309)
    planner = P.Planner(60, 24, 16)
    states = 0
    for case in range(400):
        M = rng.choice([1, 1, 2, 3, 4, 5, 8, 8, 12, 16])
        L = rng.randint(1, 60 if M <= 4 else 34)
        n_max = rng.randint(1, max(1, min(24, L)))
        n_min = rng.randint(1, n_max)
        nb = rng.choice([0, 0, rng.randint(1, 2 * L + 2), rng.randint(1, 12)])
        kw = {}
        if rng.random() < 0.15:
            kw["t_lo"] = 1 << rng.randint(20, 30)
            kw["t_hi"] = 2 * kw["t_lo"]
        if rng.random() < 0.2:
            kw["uniform_layers"] = True
        if rng.random() < 0.3:
            kw["boundary"] = rng.random() < 0.5
        var = rng.choice(["plain", "tight", "forbid"])
        inp = inputs.random_small(rng.randint(0, 10**6), L, M, n_min, n_max, nb, f=rng.randint(0, 4),
                                  tight_mem=(var == "tight"), forbid_some_d=(var == "forbid"), **kw)
        states += full_check(P, planner, inp)[1]
    planner.close()
    assert states > 1_000_000


def test_handle_reuse_across_shapes(P):
    """One handle sized for the maxima serves smaller jobs back to back."""
    planner = P.Planner(40, 6, 4)
    for i, (L, M, n_max, nb) in enumerate([(40, 4, 6, 16), (9, 2, 3, 5), (25, 3, 6, 0), (40, 1, 6, 40)]):
        full_check(P, planner, inputs.random_small(50 + i, L, M, 1, n_max, nb, f=1, tight_mem=(i % 2 == 0)))
    planner.close()


@pytest.mark.parametrize("cfg", [1, 2, 3])
def test_configs_1_to_3_every_state(P, cfg):
    inp = inputs.config(cfg)
    planner = P.Planner(inp.L, inp.n_max, inp.gpus_per_node)
    got, nstates = full_check(P, planner, inp)
    assert got["feasible"].all()
    say(f"config {cfg}: {got['states']} states ({nstates} exist), {got['candidates']} candidates: bit-exact")
    planner.close()


def check_against_golden(P, inp, path):
    g = json.load(open(path))
    planner = P.Planner(inp.L, inp.n_max, inp.gpus_per_node)
    got = planner.plan(inp)
    want = {k: np.array(v) for k, v in g.items() if isinstance(v, list)}
    want["states"], want["candidates"] = g["states"], g["candidates"]
    PU.compare_templates(got, want, inp.n_max - inp.n_min + 1)
    Smax = P.oob_plan_max_stages(inp.L, inp.n_max, inp.gpus_per_node, inp.microbatches)
    D = inp.gpus_per_node - 1 + inp.n_max
    bad = []
    for S in range(1, Smax + 1):
        h = hashlib.sha256()
        for delta in range(D):
            gb = planner.block(S, delta)
            if gb is not None:
                h.update(PU.canonical_gpu_block(gb, S, inp.L))
        if h.hexdigest() != g["level_sha256"][str(S)]:
            bad.append(S)
    planner.close()
    assert not bad, f"levels whose state records differ from the oracle's: {bad[:10]}"
    return got


@pytest.mark.timeout(900)
def test_config4_full_size_against_stored_oracle_results(P):
    """The headline workload in the configuration bench.py times.  The oracle needs minutes
    for it, so its templates and a SHA-256 per level over all state records are stored by
    tests/golden/make_golden.py (which calls only the oracle)."""
    inp = inputs.config(4)
    say("config 4 (L=98, n=8..64 x 8 GPUs)")
    got = check_against_golden(P, inp, os.path.join(GOLD, "cfg4_expected.json"))
    assert (got["states"], got["candidates"]) == (3724666, 16232508904)


@pytest.mark.timeout(900)
def test_config4_with_the_papers_microbatch_choice_against_stored_oracle_results(P):
    """Configuration 4 with N_b = 4 S' per state (the paper's planning-time choice, Section
    4.1.2): the cost coefficients then differ per level (cl = 3 r, cr = 4 s).  Stored results
    written by tests/golden/make_golden.py cfg4_paper_nb (oracle only)."""
    import dataclasses

    inp = dataclasses.replace(inputs.config(4), microbatches=0, name="cfg4_gpt175b_paper_nb")
    say("config 4, N_b = 4 S'")
    got = check_against_golden(P, inp, os.path.join(GOLD, "cfg4_paper_nb_expected.json"))
    assert (got["states"], got["candidates"]) == (3724666, 16232508904)


@pytest.mark.timeout(900)
def test_config4_repeated_calls_on_one_handle_stay_identical(P):
    """Levels run on two streams with events between them: five calls back to back on one handle
    (no host synchronisation in between) must leave exactly the stored oracle results, every
    time -- a missing dependency between the streams would show up here as a changed record."""
    import torch

    inp = inputs.config(4)
    g = json.load(open(os.path.join(GOLD, "cfg4_expected.json")))
    want = {k: np.array(v) for k, v in g.items() if isinstance(v, list)}
    want["states"], want["candidates"] = g["states"], g["candidates"]
    planner = P.Planner(inp.L, inp.n_max, inp.gpus_per_node)
    prof = P.DeviceProfile(inp)
    outs = [planner.new_outputs(inp) for _ in range(5)]
    for o in outs:
        planner.enqueue(prof, o)
    torch.cuda.synchronize()
    for i, o in enumerate(outs):
        say(f"call {i}")
        PU.compare_templates(o.to_host(), want, inp.n_max - inp.n_min + 1)
    D = inp.gpus_per_node - 1 + inp.n_max
    for S in (2, 3, 17, 50, 51, 97, 98):  # the records the last call left behind
        h = hashlib.sha256()
        for delta in range(D):
            gb = planner.block(S, delta)
            if gb is not None:
                h.update(PU.canonical_gpu_block(gb, S, inp.L))
        assert h.hexdigest() == g["level_sha256"][str(S)], S
    planner.close()


def test_call_can_be_captured_into_a_graph_and_replayed(P):
    """The call forks to the handle's second stream and joins it again with events, so a caller
    may capture it.  The graph is replayed three times with eager work in between; every replay
    must give the oracle's templates again (the output buffers are cleared before each)."""
    import torch

    inp = inputs.config(2)
    o, want = oracle_expected(inp)
    o.close()
    planner = P.Planner(inp.L, inp.n_max, inp.gpus_per_node)
    prof = P.DeviceProfile(inp)
    out = planner.new_outputs(inp)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        planner.enqueue(prof, out)  # first call: the handle creates its second stream and events
    torch.cuda.synchronize()
    PU.compare_templates(out.to_host(), want, inp.n_max - inp.n_min + 1)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        planner.enqueue(prof, out)
    for i in range(3):
        say(f"replay {i}")
        for v in out.t.values():
            v.zero_()
        torch.randn(1 << 20, device="cuda").sum().item()  # eager work and a synchronisation between replays
        graph.replay()
        torch.cuda.synchronize()
        PU.compare_templates(out.to_host(), want, inp.n_max - inp.n_min + 1)
    full = {(S, d): planner.block(S, d) for S in (2, 9, 17) for d in range(2, 8)}
    assert any(b is not None for b in full.values())
    planner.close()


def test_device_status_reports_bad_profile_values(P):
    import torch

    inp = inputs.random_small(3, 8, 2, 1, 2, 6)
    planner = P.Planner(8, 2, 2)
    bad = inputs.PlanInput("neg", inp.fwd_ns.copy(), inp.bwd_ns, inp.mem_bytes, inp.boundary_ns, 1, 2, 2, 6,
                           inp.mem_cap, 1)
    bad.fwd_ns[3, 0] = -5
    assert int(planner.plan(bad)["status"][0]) == P.OOB_EINVAL
    big = inputs.PlanInput("big", inp.fwd_ns * (1 << 45), inp.bwd_ns, inp.mem_bytes, inp.boundary_ns, 1, 2, 2,
                           6, inp.mem_cap, 1)
    assert int(planner.plan(big)["status"][0]) == P.OOB_EOVERFLOW
    assert int(planner.plan(inp)["status"][0]) == P.OOB_OK
    planner.close()


def test_large_times_stay_exact_on_both_paths(P):
    """Times near the top of the exactly representable range.  Up to a bound the set-up
    kernel checks, (total, split point) pairs fit one double and the keyed split kernel runs;
    above it the select kernel evaluates every candidate itself.  Both must match the oracle
    bit for bit."""
    planner = P.Planner(12, 4, 3)
    seen = set()
    for seed in range(4):
        for inp in (inputs.random_small(20 + seed, 9, 2, 1, 3, 7, t_lo=(1 << 38), t_hi=(1 << 39)),
                    inputs.random_small(30 + seed, 12, 3, 1, 4, 0, t_lo=(1 << 36), t_hi=(1 << 37),
                                        tight_mem=True),
                    inputs.random_small(40 + seed, 9, 2, 1, 3, 7, t_lo=(1 << 30), t_hi=(1 << 31)),
                    inputs.random_small(50 + seed, 12, 3, 1, 4, 9)):
            full_check(P, planner, inp)
            seen.add(tuple(planner.flags()[:2]))
    assert seen == {(0, 0), (1, 0)}, "keyed kernel and in-select evaluation must both have run"
    planner.close()


def test_plain_split_kernel(P):
    """The tiled split kernel without keys serves shapes whose tables exceed the keyed kernel's
    LDS classes (hundreds of nodes); the handle option routes ordinary shapes through it."""
    for inp in (inputs.config(1), inputs.config(2),
                inputs.random_small(3, 37, 3, 1, 5, 9, f=1, tight_mem=True),
                inputs.random_small(4, 30, 3, 2, 30, 0, f=2),
                inputs.random_small(21, 9, 2, 1, 3, 7, t_lo=(1 << 38), t_hi=(1 << 39))):
        print("plain", inp.name, inp.L, flush=True)
        planner = P.Planner(inp.L, inp.n_max, inp.gpus_per_node)
        planner.set_option(P.OOB_OPT_PLAIN_SPLIT, 1)
        full_check(P, planner, inp)
        assert planner.flags()[:2] == [0, 1]
        planner.close()


def test_xcd_chunked_task_order(P):
    """The other order of the workgroup tasks (block row by block row, each XCD walking one
    contiguous stretch of the list) computes the same tables."""
    for inp in (inputs.config(2), inputs.config(3),
                inputs.random_small(3, 37, 3, 1, 5, 9, f=1, tight_mem=True),
                inputs.random_small(5, 60, 2, 1, 6, 11, f=2),
                inputs.random_small(4, 30, 3, 2, 30, 0, f=2)):
        print("xcd", inp.name, inp.L, flush=True)
        planner = P.Planner(inp.L, inp.n_max, inp.gpus_per_node)
        planner.set_option(P.OOB_OPT_XCD_ORDER, 1)
        full_check(P, planner, inp)
        planner.close()


def test_select_with_eight_lanes_per_state(P):
    """The select kernel of the top levels (eight lanes per state), forced onto every level of
    shapes the oracle finishes in seconds: once reading the keys of all splits, once evaluating
    the two outer splits of every level itself (both device-set families, both N_b modes, a
    profile whose totals are too large for keys, so that its one-lane fallback runs too), the
    latter also with every launch on one stream."""
    seen = set()
    for fuse_from, one_stream in ((1 << 20, 0), (2, 0), (2, 1)):
        for inp in (inputs.config(1), inputs.config(2),
                    inputs.random_small(3, 37, 3, 1, 5, 9, f=1, tight_mem=True),
                    inputs.random_small(5, 60, 2, 1, 6, 11, f=2),
                    inputs.random_small(4, 30, 3, 2, 30, 0, f=2),
                    inputs.random_small(7, 12, 8, 1, 3, 5),
                    inputs.random_small(21, 9, 2, 1, 3, 7, t_lo=(1 << 38), t_hi=(1 << 39))):
            print("select8", fuse_from, inp.name, inp.L, flush=True)
            planner = P.Planner(inp.L, inp.n_max, inp.gpus_per_node)
            planner.set_option(P.OOB_OPT_SELECT8_FROM, 2)
            planner.set_option(P.OOB_OPT_FUSE_FROM, fuse_from)
            planner.set_option(P.OOB_OPT_ONE_STREAM, one_stream)
            full_check(P, planner, inp)
            seen.add(tuple(planner.flags()[:2]))
            planner.close()
    assert seen == {(0, 0), (1, 0)}, "keys and the evaluation without keys must both have run"


def test_two_calls_same_answer(P):
    """Determinism: the same job twice on one handle gives identical tables."""
    inp = inputs.config(2)
    planner = P.Planner(inp.L, inp.n_max, inp.gpus_per_node)
    a = planner.plan(inp)
    blocks_a = {(S, d): planner.block(S, d) for S in (2, 5, 9) for d in range(3, 12)}
    b = planner.plan(inp)
    for k in a:
        assert np.array_equal(np.asarray(a[k]), np.asarray(b[k])), k
    for (S, d), ba in blocks_a.items():
        bb = planner.block(S, d)
        assert (ba is None) == (bb is None)
        if ba is not None:
            for k in ba:
                assert np.array_equal(ba[k], bb[k])
    planner.close()
