"""Pins of the exact-minimum oracle (the dynamic program over a fixed slowest-stage time) against
exhaustive enumeration of every pipeline, and its relation to the paper's recursion.  CPU only."""
import numpy as np
import pytest

import inputs
from oracle import brute_force as bf
from oracle import capi
from oracle import exact_minimum as E


def heuristic(inp):
    r = capi.plan(inp)
    return [int(r["T"][i]) if r["feasible"][i] else None for i in range(inp.n_max - inp.n_min + 1)]


SHAPES = [(5, 1, 1, 3, 6), (6, 2, 1, 3, 8), (7, 2, 1, 2, 9), (6, 4, 1, 2, 12), (8, 4, 2, 2, 12), (6, 3, 1, 2, 7),
          (7, 1, 1, 4, 7), (8, 3, 1, 2, 8), (9, 2, 2, 3, 9)]


@pytest.mark.parametrize("shape", SHAPES)
def test_equals_exhaustive_enumeration(shape):
    """Every pipeline enumerated one by one (closed-form cost) gives the same minimum."""
    L, M, n_min, n_max, nb = shape
    for seed in range(4):
        for var in ("plain", "tight", "forbid"):
            inp = inputs.random_small(seed, L, M, n_min, n_max, nb, f=1, tight_mem=(var == "tight"),
                                      forbid_some_d=(var == "forbid"))
            got = E.exact_minimum(inp)
            for n in range(n_min, n_max + 1):
                b = bf.brute_min(inp, n)
                assert got[n - n_min] == (None if b is None else b[0]), (shape, seed, var, n)


def test_hand_case():
    """Layers (F+B) = 3, 1, 2, 2, one GPU per node, N_b = 4, worked with the closed form
    C = sum t + (N_b - S + k* - 1) t_max + sum_{k >= k*} t:
    one stage (8): 8 + 2*8 + 8 = 32; two stages: cuts after 1, 2, 3 layers cost 23, 20, 22 (the
    worked example of the recursion's pins); three stages: (3,1,4) -> 8 + 2*4 + 4 = 20,
    (3,3,2) -> 8 + 0 + 8 = 16, (4,2,2) -> 8 + 0 + 8 = 16; four stages (3,1,2,2): 8 - 3 + 8 = 13."""
    from conftest import simple_input

    inp = simple_input([3, 1, 2, 2], M=1, n_min=1, n_max=4, nb=4)
    assert E.exact_minimum(inp) == [32, 20, 16, 13]


def boundary_heavy_case():
    """Four layers of time 2 on one GPU per node; the boundary term after layer 3 is 10, the others
    0.  The stage [2, 3) costs 2 + 10 = 12, the model's last stage [2, 4) pays no boundary term and
    costs 4: a longer stage that is FASTER than the one ending a layer earlier."""
    from conftest import simple_input

    return simple_input([2, 2, 2, 2], M=1, n_min=1, n_max=3, nb=4, bnd=[0, 0, 10, 0])


def test_stage_times_are_not_monotone_in_the_last_layer():
    """Worked with C = sum t + (N_b - S + k* - 1) t_max + sum_{k >= k*} t, N_b = 4:
    one stage: t = 8: 8 + 2*8 + 8 = 32.
    two stages: (2 | 6) -> 8 + 2*6 + 6 = 26; (4 | 4) -> 8 + 1*4 + 8 = 20;
                (6+10 | 2) -> 18 + 1*16 + 18 = 52.                      minimum 20
    three stages: (2, 2, 4) -> k* = 2: 8 + 2*4 + 4 = 20; (2, 4+10, 2) -> k* = 1: 18 + 1*14 + 16 = 48;
                  (4, 2+10, 2) -> k* = 1: 18 + 1*12 + 14 = 44.          minimum 20
    A search that stops at the first too-slow stage [2, 3) (12 > tau = 4) never sees [2, 4)."""
    inp = boundary_heavy_case()
    assert E.exact_minimum(inp) == [32, 20, 20]
    for n in (1, 2, 3):
        assert bf.brute_min(inp, n)[0] == [32, 20, 20][n - 1]


def test_small_times_large_boundary_terms_against_exhaustive_enumeration():
    """Times 1..4 with boundary terms 0..5: the boundary term often exceeds a layer, so stage times
    go down when a stage grows to the model's end."""
    for seed in range(1000, 1060):
        inp = inputs.random_small(seed, 6, 2, 1, 3, 8, t_lo=1, t_hi=4)
        got = E.exact_minimum(inp)
        for n in range(1, 4):
            b = bf.brute_min(inp, n)
            assert got[n - 1] == (None if b is None else b[0]), (seed, n)


def test_never_above_the_recursion_and_gap_on_the_configurations():
    for cfg in (1, 2, 3):
        inp = inputs.config(cfg)
        exact, heur = E.exact_minimum(inp), heuristic(inp)
        gaps = []
        for e, h in zip(exact, heur):
            assert (e is None) == (h is None)
            if e is not None:
                assert e <= h
                gaps.append(h / e - 1)
        print(f"config {cfg}: recursion above the exact minimum by at most {max(gaps):.4%}, "
              f"equal for {sum(g == 0 for g in gaps)} of {len(gaps)} templates")


BINDING = {}
STAGED_SHAPES = [(5, 1, 1, 3, 6), (6, 2, 1, 3, 8), (7, 2, 1, 2, 9), (6, 4, 1, 2, 12), (6, 3, 1, 2, 7),
                 # the stage-count limit binds: N_b below min(L, n M)
                 (7, 1, 1, 4, 3), (7, 2, 1, 3, 4), (8, 2, 1, 3, 3), (6, 4, 1, 2, 3), (9, 3, 1, 2, 2),
                 # N_b = 4 S per pipeline (the paper's planning-time choice)
                 (7, 3, 1, 2, 0), (6, 2, 1, 3, 0), (8, 1, 1, 4, 0)]


@pytest.mark.parametrize("shape", STAGED_SHAPES)
def test_stage_limit_and_4S_mode_equal_exhaustive_enumeration(shape):
    """Both dynamic programs against every pipeline enumerated one by one: the one with the stage
    count in its tables always; the one without it wherever the limit cannot bind, and never above
    the exhaustive minimum (it minimises over a larger set) where it can."""
    L, M, n_min, n_max, nb = shape
    differ = 0
    for seed in range(4):
        for var in ("plain", "tight", "forbid"):
            inp = inputs.random_small(seed, L, M, n_min, n_max, nb, f=1, tight_mem=(var == "tight"),
                                      forbid_some_d=(var == "forbid"))
            staged, loose = E.exact_minimum_staged(inp), E.exact_minimum(inp, allow_bound=True)
            raw = E.unlimited_raw(inp)
            for n in range(n_min, n_max + 1):
                b = bf.brute_min(inp, n)
                b = None if b is None else b[0]
                assert staged[n - n_min] == b, (shape, seed, var, n)
                if E.is_tight(inp, n):
                    assert loose[n - n_min] == b, (shape, seed, var, n)
                else:
                    assert loose[n - n_min] == E.LIMIT_CAN_BIND
                    if b is not None:
                        assert raw[n - n_min] <= b  # a minimum over more pipelines; may even be negative
                        differ += raw[n - n_min] < b
                    else:
                        differ += raw[n - n_min] != -1  # pipelines exist only beyond the limit
    BINDING[shape] = differ


def test_the_stage_limit_changes_minima_in_those_shapes():
    """The shapes with N_b below min(L, n M) are there to test the limit: in most of them it must
    have changed at least one minimum (run after the parametrised test above)."""
    binding = [sh for sh in STAGED_SHAPES if 0 < sh[4] < min(sh[0], sh[3] * sh[1])]
    assert all(sh in BINDING for sh in binding)
    assert sum(BINDING[sh] > 0 for sh in binding) >= 3


def test_4S_mode_hand_case():
    """Layers (F+B) = 3, 1, 2, 2, one GPU per node, N_b = 4 S: C = sum t + (3 S + k* - 1) t_max + sum_{k >= k*} t.
    one stage: 8 + 2*8 + 8 = 32; two stages (4 | 4): 8 + 5*4 + 8 = 36, (3 | 5): k* = 1: 8 + 6*5 + 5 = 43,
    (6 | 2): 8 + 5*6 + 8 = 46; three stages: (3,1,4): k* = 2: 8 + 10*4 + 4 = 52, (3,3,2): 8 + 8*3 + 8 = 40,
    (4,2,2): 8 + 8*4 + 8 = 48; four stages (3,1,2,2): 8 + 11*3 + 8 = 49."""
    from conftest import simple_input

    inp = simple_input([3, 1, 2, 2], M=1, n_min=1, n_max=4, nb=0)
    assert E.exact_minimum(inp) == E.exact_minimum_staged(inp) == [32, 36, 40, 49]
    for n in range(1, 5):
        assert bf.brute_min(inp, n)[0] == [32, 36, 40, 49][n - 1]


def test_stage_limit_hand_case():
    """The same four layers with N_b = 2: pipelines of more than two stages do not exist.
    C = sum t + (2 - S + k* - 1) t_max + sum_{k >= k*} t: one stage: 8 + 0 + 8 = 16;
    two stages: (3 | 5): k* = 1: 8 + 0 + 5 = 13, (4 | 4): 8 - 4 + 8 = 12, (6 | 2): 8 - 6 + 8 = 10."""
    from conftest import simple_input

    inp = simple_input([3, 1, 2, 2], M=1, n_min=1, n_max=4, nb=2)
    assert E.exact_minimum_staged(inp) == [16, 10, None, None]
    with pytest.raises(ValueError):
        E.exact_minimum(inp)
    # without the limit three and four stages exist: those templates are marked, not answered
    assert E.exact_minimum(inp, allow_bound=True) == [16, 10, E.LIMIT_CAN_BIND, E.LIMIT_CAN_BIND]
    assert E.unlimited_raw(inp)[2] != -1 and E.unlimited_raw(inp)[3] != -1


def test_rejects_what_it_does_not_model():
    inp = inputs.random_small(0, 9, 2, 1, 3, 4)   # N_b = 4 < min(L, n_max M) = 6
    with pytest.raises(ValueError):
        E.exact_minimum(inp)
    assert E.exact_minimum(inp, allow_bound=True)[0] == E.exact_minimum_staged(inp)[0]  # n = 1: min(L, M) = 2 <= 4
