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


def test_rejects_what_it_does_not_model():
    inp = inputs.random_small(0, 9, 2, 1, 3, 4)   # N_b = 4 < min(L, n_max M) = 6
    with pytest.raises(ValueError):
        E.exact_minimum(inp)
