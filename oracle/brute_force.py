"""Exhaustive checker (test infrastructure): every explicit pipeline, closed-form cost.

A pipeline for n nodes of M GPUs is: a stage count S, cut points
0 = b_0 < b_1 < ... < b_S = L, and a GPU count per stage such that the stages,
taken in order, fill node after node exactly (no stage spans two nodes, every
GPU is used: Section 4.1.2).  Its iteration time follows from Eq. 1-4 by
induction over the recursion:

    C = sum_k t_k + (N_b - S + k* - 1) t_{k*} + sum_{k >= k*} t_k,

with t_k the stage's F+B (plus its boundary time when it is not the last
stage) and k* the first slowest stage, 0-indexed.  The recursion of the paper
keeps only one record per sub-problem, so it is a heuristic: its result is
never below the exhaustive minimum computed here and equals it whenever every
split joins two single stages.
"""
from __future__ import annotations

from itertools import combinations
from typing import Iterator, List, Optional, Sequence, Tuple

FORBIDDEN = 1 << 62


def pipeline_cost(times: Sequence[int], nb: int) -> Tuple[int, int, int, int, int]:
    """(T, T1, T2, T3, kstar) of explicit stage times under nb microbatches."""
    S = len(times)
    tmax = max(times)
    kstar = list(times).index(tmax)
    T1 = sum(times)
    T2 = (nb - S + kstar - 1) * tmax
    T3 = sum(times[kstar:])
    return T1 + T2 + T3, T1, T2, T3, kstar


def stage_time(inp, u: int, v: int, d: int) -> Optional[int]:
    """Eq. 4 plus this build's memory rule and boundary term; None = impossible."""
    t = 0
    for l in range(u, v):
        f, b = int(inp.fwd_ns[l, d - 1]), int(inp.bwd_ns[l, d - 1])
        if f >= FORBIDDEN or b >= FORBIDDEN:
            return None
        t += f + b
    total = sum(int(x) for x in inp.mem_bytes[u:v])
    if -((-total) // d) > inp.mem_cap:
        return None
    if v < inp.L:
        t += int(inp.boundary_ns[v - 1])
    return t


def _compositions(total: int, parts: int) -> Iterator[Tuple[int, ...]]:
    """All ways to write total as an ordered sum of `parts` positive integers."""
    for cuts in combinations(range(1, total), parts - 1):
        prev = 0
        out = []
        for c in cuts:
            out.append(c - prev)
            prev = c
        out.append(total - prev)
        yield tuple(out)


def gpu_assignments(n: int, M: int, S: int) -> Iterator[Tuple[int, ...]]:
    """GPU counts per stage: n nodes in order, node i holds c_i >= 1 stages whose
    GPU counts sum to M."""
    if S < n or S > n * M:
        return
    for per_node in _compositions(S, n):  # stages per node
        if any(c > M for c in per_node):
            continue

        def rec(i: int, acc: Tuple[int, ...]):
            if i == n:
                yield acc
                return
            for comp in _compositions(M, per_node[i]):
                yield from rec(i + 1, acc + comp)

        yield from rec(0, ())


def enumerate_pipelines(inp, n: int):
    """Yields (T, S, begins, gpus, times) for every feasible explicit pipeline."""
    L, M, Nb = inp.L, inp.gpus_per_node, inp.microbatches
    hi = min(L, n * M)
    if Nb > 0:
        hi = min(hi, Nb)
    for S in range(n, hi + 1):
        nb = Nb if Nb > 0 else 4 * S
        for cuts in combinations(range(1, L), S - 1):
            begins = (0,) + cuts + (L,)
            for gp in gpu_assignments(n, M, S):
                times: List[int] = []
                ok = True
                for k in range(S):
                    t = stage_time(inp, begins[k], begins[k + 1], gp[k])
                    if t is None:
                        ok = False
                        break
                    times.append(t)
                if ok:
                    yield pipeline_cost(times, nb)[0], S, begins, gp, times


def brute_min(inp, n: int):
    """Smallest cost over all explicit pipelines for n nodes, or None."""
    best = None
    for T, S, begins, gp, times in enumerate_pipelines(inp, n):
        if best is None or T < best[0]:
            best = (T, S, begins, gp, times)
    return best


def representable_counts(sizes: Sequence[int], target: int) -> List[int]:
    """All pipeline counts sum(x_i) over non-negative x with sum(x_i * size_i) = target
    (plain recursive enumeration, for the coverage tests)."""
    sizes = sorted(sizes)
    out = set()

    def rec(idx: int, remaining: int, used: int):
        if remaining == 0:
            out.add(used)
            return
        if idx == len(sizes):
            return
        c = 0
        while c * sizes[idx] <= remaining:
            rec(idx + 1, remaining - c * sizes[idx], used + c)
            c += 1

    rec(0, target, 0)
    return sorted(out)
