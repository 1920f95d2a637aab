"""CPU oracle (test infrastructure only): the exact minimum of the pipeline cost of Section 4.1.2
over all explicit pipelines of a template, by the dynamic program of oob_exact_oracle.c (fixed
slowest-stage time tau, separable prefix and suffix).  The paper's recursion (Eq. 1-3) is a
heuristic for this minimum; the difference is its optimality gap."""
from __future__ import annotations

import ctypes as C
from typing import List, Optional

import numpy as np

from . import capi


def exact_minimum(inp) -> List[Optional[int]]:
    """Exact minimum cost for n = n_min .. n_max nodes (None where no pipeline exists).
    Needs N_b >= min(L, n_max M): the limit S <= N_b is not modelled."""
    lib = capi.lib()
    i64p = C.POINTER(C.c_int64)
    lib.oob_oracle_exact_minimum.argtypes = [i64p, i64p, i64p, i64p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                             C.c_int64, i64p]
    lib.oob_oracle_exact_minimum.restype = C.c_int64
    arrs = [np.ascontiguousarray(a, dtype=np.int64) for a in (inp.fwd_ns, inp.bwd_ns, inp.mem_bytes, inp.boundary_ns)]
    best = np.zeros(inp.n_max - inp.n_min + 1, dtype=np.int64)
    rc = lib.oob_oracle_exact_minimum(*[a.ctypes.data_as(i64p) for a in arrs], inp.L, inp.gpus_per_node, inp.n_min,
                                      inp.n_max, inp.microbatches, inp.mem_cap, best.ctypes.data_as(i64p))
    if rc < 0:
        raise ValueError("exact_minimum: needs N_b >= min(L, n_max M) and positive dimensions")
    return [None if v < 0 else int(v) for v in best]
