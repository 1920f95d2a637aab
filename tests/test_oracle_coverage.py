"""Node specification (Section 4.1.1) and coverage (Appendix A) of the CPU oracle."""
import json
import os

import numpy as np
import pytest

from oracle import brute_force as bf
from oracle import capi

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_paper_example_13_nodes():
    g = json.load(open(os.path.join(GOLD, "coin_examples.json")))
    sizes, target = g["sizes"], g["target"]
    for comb in g["combinations"]:
        assert sum(x * n for x, n in zip(comb, sizes)) == target
        assert sum(comb) in bf.representable_counts(sizes, target)
    # templates 2,3,4 feasible, f chosen so that N = n_hi + f*n0 = 4 + f*2 >= 13 -> f = 5
    feasible = np.array([1, 1, 1], dtype=np.int32)
    c = capi.coverage(feasible, 2, 5)
    n0, n_hi, p, N, cond, lo, thm, tail = c["hdr"].tolist()
    assert (n0, n_hi, p, N, cond) == (2, 4, 3, 14, 1)
    assert lo == min(12, 9)
    # 13 nodes: at most 6 pipelines (5 of size 2 and one of size 3)
    assert c["maxpipes"][13 - lo] == max(bf.representable_counts(sizes, 13)) == 6


@pytest.mark.parametrize("n0", [1, 2, 3, 5, 8])
@pytest.mark.parametrize("extra", [0, 1, 4])
@pytest.mark.parametrize("f", [0, 1, 3])
def test_theorem_a_brute_force(n0, extra, f):
    """p > n0 - 1 consecutive sizes: every N' in [(f+1) n0, N] is a sum with at
    least f+1 pipelines; checked by plain enumeration."""
    p = n0 + extra  # > n0 - 1
    n_min = max(1, n0 - 2)
    feasible = np.zeros(n0 - n_min + p + 2, dtype=np.int32)
    feasible[n0 - n_min: n0 - n_min + p] = 1  # infeasible below n0, a gap after n_hi
    c = capi.coverage(feasible, n_min, f)
    h = c["hdr"].tolist()
    n_hi = n0 + p - 1
    N = n_hi + f * n0
    assert h[:5] == [n0, n_hi, p, N, 1]
    lo = h[5]
    assert lo == min((f + 1) * n0, max(1, N - f))
    sizes = list(range(n0, n_hi + 1))
    for x in range(lo, N + 1):
        counts = bf.representable_counts(sizes, x)
        want = max(counts) if counts else 0
        assert c["maxpipes"][x - lo] == want
        if x >= (f + 1) * n0:
            assert want >= f + 1
    assert h[6] == 1


def test_condition_fails_when_too_few_sizes():
    """sizes {4,5}: p = 2 <= n0 - 1 = 3; N' = 11 = (f+1) n0 + 3 with f = 1 is not
    a sum of 4s and 5s."""
    feasible = np.array([1, 1, 0, 1], dtype=np.int32)  # run stops at the first gap
    c = capi.coverage(feasible, 4, 1)
    h = c["hdr"].tolist()
    assert h[:5] == [4, 5, 2, 9, 0]
    # range [8, 9]: 8 = 4+4, 9 = 4+5 -> covered here although the condition fails
    assert h[6] == 1
    c = capi.coverage(np.array([1, 1], dtype=np.int32), 4, 3)  # N = 5 + 12 = 17, range [16, 17]
    assert c["hdr"].tolist()[6] == 1
    # a case where it really fails: sizes {5, 6}, f = 2 -> N = 16, range [15, 16]: 16 = 5+5+6 ok;
    c = capi.coverage(np.array([1, 1], dtype=np.int32), 5, 2)
    lo = c["hdr"][5]
    for x in range(int(lo), int(c["hdr"][3]) + 1):
        counts = bf.representable_counts([5, 6], x)
        assert c["maxpipes"][x - lo] == (max(counts) if counts else 0)


def test_no_feasible_template():
    c = capi.coverage(np.zeros(4, dtype=np.int32), 1, 2)
    assert c["hdr"].tolist() == [0] * 8 and not c["maxpipes"].any()


def test_tail_range_n_minus_f():
    """Every node count from N - f to N is a sum of the chosen sizes when the run of
    sizes is long enough (here n0 = 1)."""
    c = capi.coverage(np.ones(4, dtype=np.int32), 1, 1)  # config-1 shape: sizes 1..4, f = 1
    assert c["hdr"].tolist() == [1, 4, 4, 5, 1, 2, 1, 1]
    assert c["maxpipes"][:4].tolist() == [2, 3, 4, 5]
