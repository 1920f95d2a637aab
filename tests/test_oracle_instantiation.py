"""Pins of the instantiation-enumeration oracle (Section 4.2.1, Eq. 5): the paper's worked
example, the plain definition by exhaustive search, partition numbers, the list order, and the
two evaluations (table of lists / top-down C) against each other."""
import json
import os
import random

import numpy as np
import pytest

from oracle import instantiation as I

GOLD = os.path.join(os.path.dirname(__file__), "golden", "instantiation_examples.json")


def test_paper_example_sizes_2_3_4():
    g = json.load(open(GOLD))
    sizes = g["sizes"]
    thirteen = I.instantiations(sizes, 13, 0)
    for v in g["thirteen_contains"]:
        assert tuple(v) in thirteen
    # the figure: X(3, 7) = copy of X(2, 7), then X(3, 3) with one more four-node pipeline
    want = [tuple(v) for v in g["seven_copy_of_X_2_7"] + g["seven_theta_of_X_3_3"]]
    assert I.instantiations(sizes, 7, 0) == want
    X = I.table_of_lists(sizes, 7)
    assert X[2][7] == [tuple(v) for v in g["seven_copy_of_X_2_7"]]
    assert X[3][3] == [(0, 1, 0)]
    assert all(sum(a * n for a, n in zip(v, sizes)) == 13 for v in thirteen)


def random_sizes(rng, p, hi):
    return sorted(rng.sample(range(1, hi + 1), p))


def test_equals_the_plain_definition_on_small_cases():
    rng = random.Random(5)
    for _ in range(60):
        p = rng.randint(1, 5)
        sizes = random_sizes(rng, p, 9)
        N, f = rng.randint(0, 24), rng.randint(0, 4)
        got = I.instantiations(sizes, N, f)
        assert len(set(got)) == len(got)          # no vector twice
        assert set(got) == I.exhaustive(sizes, N, f), (sizes, N, f)


def test_list_order_is_colexicographic():
    """Eq. 5 puts every vector with x_{p-1} = 0 first (the copy of X(p-1, N)), then x_{p-1} = 1,
    ...; inside each group the same rule applies to x_{p-2}: ascending order, last count first."""
    rng = random.Random(6)
    for _ in range(30):
        sizes = random_sizes(rng, rng.randint(1, 5), 8)
        N, f = rng.randint(1, 26), rng.randint(0, 3)
        got = I.instantiations(sizes, N, f)
        assert got == sorted(I.exhaustive(sizes, N, f), key=lambda v: v[::-1])


def test_counts_are_partition_numbers_when_every_size_is_a_template():
    # p(n): partitions of n (textbook values)
    for n, pn in ((1, 1), (5, 7), (10, 42), (20, 627), (30, 5604), (40, 37338)):
        count, allc = I.instantiations_c(list(range(1, n + 1)), n, 0, count_only=True)
        assert allc == pn
        assert count == pn          # f = 0: one pipeline suffices
    # at least k parts: p(n) minus partitions into fewer than k parts; k = 2 excludes only (n)
    assert I.instantiations_c(list(range(1, 21)), 20, 1, count_only=True)[0] == 627 - 1
    # partitions of 10 into at least 3 parts = 42 - 1 - 5
    assert I.instantiations_c(list(range(1, 11)), 10, 2, count_only=True)[0] == 36


def test_c_evaluation_equals_table_of_lists_order_included():
    rng = random.Random(7)
    for _ in range(40):
        sizes = random_sizes(rng, rng.randint(1, 6), 10)
        N, f = rng.randint(0, 30), rng.randint(0, 5)
        want = I.instantiations(sizes, N, f)
        got, allc = I.instantiations_c(sizes, N, f)
        assert [tuple(int(a) for a in row) for row in got] == want
        assert allc == len(I.table_of_lists(sizes, N)[len(sizes)][N])


def test_filter_and_degenerate_cases():
    assert I.instantiations((2, 3), 0, 0) == []            # the empty set has no pipeline
    assert I.instantiations((2, 3), 1, 0) == []            # not representable
    assert I.instantiations((5,), 15, 2) == [(3,)]
    assert I.instantiations((5,), 15, 3) == []             # needs four pipelines, only three fit
    got = I.instantiations((1, 2), 4, 2)                   # at least three pipelines
    assert got == [(4, 0), (2, 1)]
    off, v = I.instantiations_range((2, 3, 4), 6, 8, 1)
    assert off.tolist() == [0, 3, 5, 9] and v.shape == (9, 3)   # 6: 3 ways, 7: 2, 8: 4 (by hand)
    assert all(int(r[0]) * 2 + int(r[1]) * 3 + int(r[2]) * 4 == 8 for r in v[5:])


def test_headline_workload_counts():
    """Templates for 8..64 nodes, f = 8: every N' from (f+1) n0 = 72 to N = 128."""
    sizes = list(range(8, 65))
    count, allc = I.instantiations_c(sizes, 128, 8, count_only=True)
    assert (count, allc) == (165565, 489017)
    # a vector with fewer than nine pipelines of >= 8 nodes cannot be dropped below 72 nodes
    assert I.instantiations_c(sizes, 72, 8, count_only=True)[0] == 1   # nine 8-node pipelines
