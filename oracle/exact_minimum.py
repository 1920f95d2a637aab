"""CPU oracle (test infrastructure only): the exact minimum of the pipeline cost of Section 4.1.2
over all explicit pipelines of a template, by the dynamic programs of oob_exact_oracle.c (fixed
slowest-stage time tau, separable prefix and suffix).  The paper's recursion (Eq. 1-3) is a
heuristic for this minimum; the difference is its optimality gap.

`exact_minimum` keeps no stage count: exact for a template n when the limit S <= N_b cannot bind
(N_b = 0, the paper's N_b = 4 S per pipeline, or N_b >= min(L, n M)); for the other templates it
reports LIMIT_CAN_BIND instead of a number (the minimum over the larger set of pipelines is only a
lower bound, and with more stages than microbatches the cost formula even turns negative).
`exact_minimum_staged` carries the stage count in its tables and is exact for every N_b (small
and middle sizes only: its tables are (L+1) (n_max M + 1) (S_max + 1) entries per thread)."""
from __future__ import annotations

import ctypes as C
from typing import List, Optional

import numpy as np

from . import capi


LIMIT_CAN_BIND = -2  # same marker as the C boundary of the HIP path uses


def is_tight(inp, n: int) -> bool:
    """Whether the minimum without the stage-count limit is the exact minimum for n nodes."""
    return inp.microbatches == 0 or inp.microbatches >= min(inp.L, n * inp.gpus_per_node)


def _raw(name: str, inp) -> List[int]:
    lib = capi.lib()
    i64p = C.POINTER(C.c_int64)
    fn = getattr(lib, name)
    fn.argtypes = [i64p, i64p, i64p, i64p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int64, i64p]
    fn.restype = C.c_int64
    arrs = [np.ascontiguousarray(a, dtype=np.int64) for a in (inp.fwd_ns, inp.bwd_ns, inp.mem_bytes, inp.boundary_ns)]
    best = np.zeros(inp.n_max - inp.n_min + 1, dtype=np.int64)
    rc = fn(*[a.ctypes.data_as(i64p) for a in arrs], inp.L, inp.gpus_per_node, inp.n_min, inp.n_max, inp.microbatches,
            inp.mem_cap, best.ctypes.data_as(i64p))
    if rc < 0:
        raise ValueError(f"{name}: bad arguments")
    return [int(v) for v in best]


def _call(name: str, inp) -> List[Optional[int]]:
    return [None if v < 0 else v for v in _raw(name, inp)]


def unlimited_raw(inp) -> List[int]:
    """The numbers of the dynamic program without the stage count as it returns them (-1: no pipeline),
    also for templates whose limit can bind: there they are lower bounds of the minimum under the
    limit and can be negative (the coefficient N_b - S + k* - 1 of the slowest stage is)."""
    return _raw("oob_oracle_exact_minimum", inp)


def exact_minimum(inp, allow_bound: bool = False) -> List[Optional[int]]:
    """Minimum cost for n = n_min .. n_max nodes without the stage-count limit (None where no
    pipeline exists).  Raises unless it is the exact minimum for every template; with allow_bound the
    templates whose limit can bind get LIMIT_CAN_BIND instead."""
    tight = [is_tight(inp, n) for n in range(inp.n_min, inp.n_max + 1)]
    if not allow_bound and not all(tight):
        raise ValueError("exact_minimum: the limit S <= N_b can bind (N_b < min(L, n_max M)); "
                         "use exact_minimum_staged, or allow_bound=True for the templates it cannot bind for")
    return [v if ok else LIMIT_CAN_BIND for v, ok in zip(_call("oob_oracle_exact_minimum", inp), tight)]


def exact_minimum_staged(inp) -> List[Optional[int]]:
    """Exact minimum cost for n = n_min .. n_max nodes under S <= N_b (N_b = 0: N_b = 4 S)."""
    return _call("oob_oracle_exact_minimum_staged", inp)
