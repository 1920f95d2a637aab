"""The entry point for callers that cannot allocate (oob_inst_enumerate_static: the count table in a
static device array of the library) against the two-call form with a caller's workspace, through
the C ABI: identical offsets, vectors and status, on calls in a row that share the array."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import torch
    import paper_2309_08125_amd as pkg

    assert torch.cuda.is_available()
    pkg.load()
    return pkg


def both_ways(P, sizes, N_lo, N_hi, f, n0=0, p=0, capacity=None):
    """(offsets, vectors, status) from oob_inst_count + oob_inst_enumerate, and from the static form."""
    import torch

    inst = P.Instantiator(sizes, N_lo, N_hi, f, n0=n0, p=p)
    off, want, st = inst.enumerate()
    assert st == P.OOB_OK
    total = int(off[-1])
    cap = total if capacity is None else capacity
    dev = inst.device
    x = torch.full((inst.p, max(cap, 1)), 0x7777, dtype=torch.int16, device=dev)
    offsets = torch.full((N_hi - N_lo + 2,), -1, dtype=torch.int64, device=dev)
    status = torch.full((1,), -99, dtype=torch.int32, device=dev)
    s = torch.cuda.current_stream(dev)
    rc = P.oob_inst_enumerate_static(inst.sizes.data_ptr() if inst.sizes is not None else 0, inst.p, n0, N_lo, N_hi, f,
                                     x.data_ptr(), cap, offsets.data_ptr(), status.data_ptr(), s.cuda_stream)
    assert rc == P.OOB_OK
    torch.cuda.synchronize(dev)
    return off, want, offsets.cpu().numpy(), x.cpu().numpy().view("uint16"), int(status.item()), total


def test_static_form_equals_the_workspace_form_on_calls_in_a_row(P):
    # the headline node specification first (sizes 8..64, f = 8, 72..128 nodes: 1 343 380 vectors, a table
    # of 1 MB), then smaller inputs that reuse the same array: a list of sizes, the paper's (2, 3, 4)
    # example, and an input with no feasible vector at all
    cases = [dict(sizes=None, N_lo=72, N_hi=128, f=8, n0=8, p=57),
             dict(sizes=list(range(90, 130, 3)), N_lo=1000, N_hi=1100, f=2),
             dict(sizes=[2, 3, 4], N_lo=0, N_hi=13, f=0),
             dict(sizes=None, N_lo=20, N_hi=48, f=4, n0=4, p=26),
             dict(sizes=[5, 7], N_lo=1, N_hi=4, f=0)]
    for c in cases:
        print("case", {k: (v if k != "sizes" or v is None else f"{len(v)} sizes") for k, v in c.items()}, flush=True)
        off, want, off2, x2, st2, total = both_ways(P, **c)
        assert st2 == P.OOB_OK
        assert np.array_equal(off, off2)
        assert np.array_equal(x2[:, :total].T, want)
    assert total == 0


def test_static_form_capacity_and_limits(P):
    import torch

    # total exceeds the capacity: status on the device, offsets valid, nothing written
    off, want, off2, x2, st2, total = both_ways(P, [2, 3, 4], 0, 13, 0, capacity=5)
    assert total > 5 and st2 == P.OOB_ECAPACITY and np.array_equal(off, off2) and (x2 == 0x7777).all()
    # a table beyond the static array is refused on the host, before anything is enqueued
    assert P.oob_inst_workspace_size(1023, 4095, 0) > P.OOB_INST_STATIC_BYTES
    fake = 0x10000
    assert P.oob_inst_enumerate_static(0, 1023, 3073, 3990, 4095, 0, fake, 10, fake, fake, 0) == P.OOB_ECAPACITY
    assert P.oob_inst_enumerate_static(0, 0, 1, 0, 10, 0, fake, 10, fake, fake, 0) == P.OOB_EINVAL
    assert P.oob_inst_enumerate_static(0, 3, 2, 0, 10, 0, fake, 10, 0, fake, 0) == P.OOB_EINVAL
    # bad sizes: status OOB_EINVAL from the counting kernel, as in the workspace form
    dev = torch.device("cuda:0")
    sizes = torch.tensor([3, 3, 4], dtype=torch.int32, device=dev)
    offsets = torch.full((14,), -1, dtype=torch.int64, device=dev)
    status = torch.full((1,), -99, dtype=torch.int32, device=dev)
    x = torch.zeros((3, 8), dtype=torch.int16, device=dev)
    s = torch.cuda.current_stream(dev)
    assert P.oob_inst_enumerate_static(sizes.data_ptr(), 3, 0, 0, 12, 0, x.data_ptr(), 8, offsets.data_ptr(),
                                       status.data_ptr(), s.cuda_stream) == P.OOB_OK
    torch.cuda.synchronize(dev)
    assert int(status.item()) == P.OOB_EINVAL and not offsets.cpu().numpy().any()
