"""Instantiation enumeration (Section 4.2.1, Eq. 5) through the C ABI against the CPU oracle:
every vector, in list order, bit for bit (integer work: no tolerance)."""
import random

import numpy as np
import pytest

from oracle import instantiation as I

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import torch
    import paper_2309_08125_amd as pkg

    assert torch.cuda.is_available()
    pkg.load()
    return pkg


def compare(P, sizes, N_lo, N_hi, f, consecutive=None):
    if consecutive is None:
        inst = P.Instantiator(sizes, N_lo, N_hi, f)
    else:
        n0, p = consecutive
        sizes = list(range(n0, n0 + p))
        inst = P.Instantiator(None, N_lo, N_hi, f, n0=n0, p=p)
    off, x, st = inst.enumerate()
    want_off, want = I.instantiations_range(sizes, N_lo, N_hi, f)
    assert st == P.OOB_OK
    assert np.array_equal(off, want_off), (sizes, N_lo, N_hi, f)
    assert x.shape == want.shape and np.array_equal(x, want), (sizes, N_lo, N_hi, f)
    return len(want)


def test_paper_example_and_degenerate_cases(P):
    print("sizes (2,3,4)", flush=True)
    assert compare(P, [2, 3, 4], 0, 13, 0) > 0
    assert compare(P, [2, 3, 4], 13, 13, 0) == 5
    assert compare(P, [2, 3, 4], 7, 7, 0) == 2
    assert compare(P, [5], 15, 15, 3) == 0        # empty list: nothing to write
    assert compare(P, [5], 0, 0, 0) == 0          # no node, no pipeline
    assert compare(P, [1], 0, 9, 4) == 5          # one size: one vector per N' >= 5
    assert compare(P, [7, 9], 1, 6, 0) == 0       # nothing representable


def test_random_size_lists(P):
    rng = random.Random(11)
    for case in range(40):
        p = rng.randint(1, 9)
        sizes = sorted(rng.sample(range(1, 16), p))
        N_lo = rng.randint(0, 30)
        N_hi = N_lo + rng.randint(0, 25)
        f = rng.randint(0, 7)
        print(f"case {case}: sizes {sizes} N' {N_lo}..{N_hi} f {f}", flush=True)
        compare(P, sizes, N_lo, N_hi, f)


@pytest.mark.parametrize("n0,n_hi,f", [(1, 4, 1), (2, 16, 3), (4, 32, 4), (1, 32, 8), (8, 64, 8)])
def test_node_specifications_of_the_planning_workloads(P, n0, n_hi, f):
    """Consecutive sizes n0..n_hi, every N' from (f+1) n0 to N = n_hi + f n0 (Section 4.1.1):
    the five planning configurations; the last is the headline one (57 sizes, 1 343 380 vectors
    over several thousand wave-sized pieces with a ragged tail)."""
    N = n_hi + f * n0
    print(f"n0 {n0} n_hi {n_hi} f {f} N {N}", flush=True)
    total = compare(P, None, (f + 1) * n0, N, f, consecutive=(n0, n_hi - n0 + 1))
    if (n0, n_hi, f) == (8, 64, 8):
        assert total == 1343380


def test_large_cluster_sizes_take_the_table_from_global_memory(P):
    """Two planes of the count table exceed the LDS here: the counting kernel's other path."""
    print("sizes 500,700,900", flush=True)
    assert compare(P, [500, 700, 900], 1900, 2000, 3) > 0
    sizes = list(range(90, 130, 3))
    print("sizes", sizes, flush=True)
    assert compare(P, sizes, 1000, 1100, 2) > 1000


def test_largest_dimensions_the_entry_points_take(P):
    """OOB_INST_MAX_P template sizes and cluster sizes up to OOB_INST_MAX_N: 1023 sizes
    3073..4095, N' = 3990..4095: one pipeline of exactly N' nodes is the only way each time."""
    sizes = list(range(3073, 4096))
    print("1023 sizes, N' 3990..4095", flush=True)
    assert compare(P, sizes, 3990, 4095, 0) == 106
    assert compare(P, sizes, 4000, 4095, 1) == 0          # two pipelines never fit


def test_integer_table_path(P):
    """Counts of 2^53 and more keep the table in int64 (no case the oracle could enumerate gets
    there): the test hook forces that path on ordinary cases."""
    lib = P.load()
    assert lib.oob_inst_keep_wide_table(1) == 0
    try:
        assert compare(P, [2, 3, 4], 0, 13, 0) > 0
        assert compare(P, None, 20, 48, 4, consecutive=(4, 29)) == 10251
        assert compare(P, list(range(90, 130, 3)), 1000, 1100, 2) > 1000
    finally:
        assert lib.oob_inst_keep_wide_table(0) == 1


def test_status_codes_and_capacity(P):
    import torch

    inst = P.Instantiator([3, 3, 4], 0, 12, 0)          # not strictly increasing
    off, st = inst.count()
    assert st == P.OOB_EINVAL and not off.any()
    inst = P.Instantiator([0, 2], 0, 12, 0)             # not positive
    assert inst.count()[1] == P.OOB_EINVAL
    inst = P.Instantiator(list(range(1, 31)), 30, 30, 0)
    off, st = inst.count()
    assert st == P.OOB_OK and int(off[-1]) == 5604       # partitions of 30
    x = torch.full((30, 100), 7777, dtype=torch.int16, device="cuda")
    inst.enqueue(x, 100)                                 # too small: nothing may be written
    torch.cuda.synchronize()
    assert int(inst.status.item()) == P.OOB_ECAPACITY
    assert bool((x.cpu() == 7777).all())
    assert int(inst.offsets[-1].item()) == 5604
    # lists longer than 2^62 are reported, not enumerated
    inst = P.Instantiator(None, 1000, 1000, 0, n0=1, p=200)   # partitions of 1000 into parts <= 200
    assert inst.count()[1] == P.OOB_EOVERFLOW


def test_capacity_larger_than_total_leaves_the_tail_untouched(P):
    import torch

    inst = P.Instantiator([2, 3, 4], 13, 13, 0)
    assert inst.count()[1] == P.OOB_OK
    x = torch.full((3, 64), 7777, dtype=torch.int16, device="cuda")
    inst.enqueue(x, 64)
    torch.cuda.synchronize()
    h = x.cpu().numpy()
    assert int(inst.status.item()) == P.OOB_OK
    assert h[:, :5].T.tolist() == [[5, 1, 0], [2, 3, 0], [3, 1, 1], [0, 3, 1], [1, 1, 2]]
    assert (h[:, 5:] == 7777).all()
