import os
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # the tests load the library that is built; they compile it only if there is none
    from paper_2309_08125_amd import build as hip_build

    hip_build.ensure_built()


def simple_input(fb, M=1, n_min=1, n_max=1, nb=4, cap=None, f=0, mem=None, bnd=None,
                 fb_by_d=None):
    """PlanInput from a list of per-layer F+B values (F = fb, B = 0).

    fb_by_d: optional [L][M] table of F+B per GPU count; default divides by d
    rounding up."""
    from inputs import PlanInput

    L = len(fb)
    fwd = np.zeros((L, M), dtype=np.int64)
    bwd = np.zeros((L, M), dtype=np.int64)
    for l in range(L):
        for d in range(1, M + 1):
            fwd[l, d - 1] = fb_by_d[l][d - 1] if fb_by_d is not None else -((-fb[l]) // d)
    mem = np.array(mem if mem is not None else [1] * L, dtype=np.int64)
    bnd = np.array(bnd if bnd is not None else [0] * L, dtype=np.int64)
    if cap is None:
        cap = int(mem.sum()) + 1
    return PlanInput("simple", fwd, bwd, mem, bnd, n_min, n_max, M, nb, cap, f)


@pytest.fixture
def make_simple():
    return simple_input
