"""CPU oracle (test infrastructure only) of the instantiation enumeration, Section 4.2.1, Eq. 5.

`table_of_lists` is the dynamic program exactly as the paper draws it: a table with one cell per
(p', N') that holds the LIST of count vectors X(p', N'), filled from cell (0, 0) upwards with

    X(p', N') = X(p'-1, N')  ++  theta(X(p', N' - n_{p'-1}), p'-1)

(p' = number of template sizes in play; theta adds one to x_{p'-1} of every vector), followed
by the filter "at least f+1 pipelines" on the bottom-right cell.  Slow and memory hungry on
purpose; `oob_inst_oracle.c` evaluates the same equation top-down for the large cases and is
pinned against this one.  `exhaustive` is the plain definition (every vector of bounded
counts, tested one by one) used to pin both.
"""
from __future__ import annotations

import ctypes as C
import itertools
from typing import List, Sequence, Tuple

import numpy as np

Vector = Tuple[int, ...]


def theta(vectors: List[Vector], j: int) -> List[Vector]:
    return [v[:j] + (v[j] + 1,) + v[j + 1:] for v in vectors]


def table_of_lists(sizes: Sequence[int], N: int) -> List[List[List[Vector]]]:
    p = len(sizes)
    X = [[[] for _ in range(N + 1)] for _ in range(p + 1)]
    X[0][0] = [tuple([0] * p)]
    for pp in range(1, p + 1):
        n = sizes[pp - 1]
        for Np in range(N + 1):
            second = theta(X[pp][Np - n], pp - 1) if Np >= n else []
            X[pp][Np] = X[pp - 1][Np] + second
    return X


def instantiations(sizes: Sequence[int], N: int, f: int) -> List[Vector]:
    """Feasible pipeline sets for N nodes: requirement 1 by Eq. 5, requirement 2 by the filter."""
    return [v for v in table_of_lists(sizes, N)[len(sizes)][N] if sum(v) >= f + 1]


def exhaustive(sizes: Sequence[int], N: int, f: int) -> set:
    ranges = [range(N // n + 1) for n in sizes]
    return {v for v in itertools.product(*ranges)
            if sum(a * n for a, n in zip(v, sizes)) == N and sum(v) >= f + 1}


def instantiations_c(sizes: Sequence[int], N: int, f: int, count_only: bool = False):
    """The C evaluation of Eq. 5: (array [count, p] of uint16 in list order, |X(p, N)|)."""
    from . import capi

    lib = capi.lib()
    s = np.ascontiguousarray(sizes, dtype=np.int32)
    sp = s.ctypes.data_as(C.POINTER(C.c_int32))
    allc = C.c_int64(0)
    n = lib.oob_oracle_instantiate(sp, len(s), N, f, None, 0, C.byref(allc))
    if count_only:
        return n, allc.value
    out = np.zeros((n, len(s)), dtype=np.uint16)
    lib.oob_oracle_instantiate(sp, len(s), N, f, out.ctypes.data_as(C.POINTER(C.c_uint16)), n, C.byref(allc))
    return out, allc.value


def instantiations_range(sizes: Sequence[int], N_lo: int, N_hi: int, f: int):
    """All N' in [N_lo, N_hi]: (offsets [N_hi - N_lo + 2], vectors [total, p]) in N' order."""
    parts = [instantiations_c(sizes, Np, f)[0] for Np in range(N_lo, N_hi + 1)]
    off = np.zeros(len(parts) + 1, dtype=np.int64)
    off[1:] = np.cumsum([len(a) for a in parts])
    return off, (np.concatenate(parts, axis=0) if parts else np.zeros((0, len(sizes)), np.uint16))
