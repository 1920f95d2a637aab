"""CPU oracle (test infrastructure only) of the batch distribution, Section 4.2.2, Eq. 6, and of
the choice between instantiation vectors by throughput that it serves.

Eq. 6: pipeline i of the x pipelines of a plan gets N_i microbatches; with T_i the time of one
microbatch in pipeline i, the plan minimises  sum_i (N_i T_i - mean)^2  under  sum_i N_i b = B.
The paper hands this to a general integer solver, so the only thing an oracle can follow is the
definition: `exhaustive` tries every vector N.  `sweep` reaches the same minimum by a different
route (below) and serves as the second evaluation that pins the first, and as the method for
sizes the definition cannot reach.

Readings (the paper leaves these open or prints them inconsistently):
  * the unknowns are per pipeline (the objective's index set); the constraint's sum is read as
    sum_i N_i = Q = B / b over the same pipelines.  Pipelines of one template have equal T, and
    an optimum gives them counts that differ by at most one;
  * N_i >= 1: every pipeline holds a replica and takes part in the iteration, so a batch with
    Q < x microbatches cannot be distributed (the case in which the paper recommends another
    batch size);
  * all arithmetic is in integers: x * sum_i (N_i T_i - mean)^2 = x sum a_i^2 - (sum a_i)^2,
    a_i = N_i T_i, is what is minimised and reported (`vx`);
  * several N can reach the minimum (always so for pipelines of equal T); the minimum is
    unique, the vector is not: `exhaustive` returns all of them;
  * throughput of a plan = B / (time of its slowest pipeline) = B / max_i N_i T_i, the linear
    model of Eq. 6 itself; between plans of equal time the first in list order wins.

`sweep`: for a fixed level mu the problem  min sum_i (N_i T_i - mu)^2  is a separable convex
allocation, for which "no exchange of one microbatch between two pipelines improves it" is
optimality, and as mu grows its optimum changes by such single exchanges, each at a level that
is a ratio of integers.  Every allocation on this path is feasible for Eq. 6, and the path
passes an allocation that is optimal for Eq. 6 when mu is that optimum's own mean (the value of
sum (a_i - mu)^2 at the mean IS the variance, and no N has a smaller one).  So the smallest
variance met along the path from mu = 0 to mu = Q max T is the minimum of Eq. 6.
"""
from __future__ import annotations

from fractions import Fraction
from typing import List, Optional, Sequence, Tuple


def vx(T: Sequence[int], N: Sequence[int]) -> int:
    """x * sum_i (N_i T_i - mean)^2 as an exact integer."""
    a = [n * t for n, t in zip(N, T)]
    return len(a) * sum(v * v for v in a) - sum(a) ** 2


def exhaustive(T: Sequence[int], Q: int) -> Tuple[Optional[int], List[List[int]]]:
    """The definition: every N with N_i >= 1 and sum N_i = Q.  (minimum of vx, all its minimisers
    in lexicographic order); (None, []) when Q < x."""
    x = len(T)
    best: Optional[int] = None
    arg: List[List[int]] = []

    def rec(i: int, left: int, cur: List[int]) -> None:
        nonlocal best, arg
        if i == x - 1:
            N = cur + [left]
            v = vx(T, N)
            if best is None or v < best:
                best, arg = v, [N]
            elif v == best:
                arg.append(N)
            return
        for n in range(1, left - (x - 1 - i) + 1):
            rec(i + 1, left - n, cur + [n])

    if 1 <= x <= Q:
        rec(0, Q, [])
    return best, arg


def allocation_at(T: Sequence[int], Q: int, mu: Fraction) -> List[int]:
    """An optimum of  min sum_i (N_i T_i - mu)^2, sum N_i = Q, N_i >= 1  by marginal allocation
    (exact for separable convex costs): one microbatch at a time to where it costs least."""
    x = len(T)
    N = [1] * x
    for _ in range(Q - x):
        j = min(range(x), key=lambda j: (T[j] * T[j] + 2 * T[j] * T[j] * N[j] - 2 * T[j] * mu, j))
        N[j] += 1
    return N


def sweep(T: Sequence[int], Q: int) -> Tuple[Optional[int], Optional[List[int]], int]:
    """(minimum of vx, one minimiser, exchanges made) by following the optimal allocation of the
    fixed-level problem from mu = 0 to mu = Q max T."""
    x = len(T)
    if not 1 <= x <= Q:
        return None, None, 0
    mu, mu_end = Fraction(0), Fraction(Q * max(T))
    N = allocation_at(T, Q, mu)
    best, arg, steps = vx(T, N), list(N), 0
    while True:
        nxt = None
        for i in range(x):           # a microbatch leaves pipeline i ...
            if N[i] < 2:
                continue
            for j in range(x):       # ... for pipeline j: gain(mu) = c - 2 mu (T_j - T_i)
                if T[i] >= T[j]:     # the gain of such an exchange does not grow with mu: N is optimal at
                    continue         # mu, so it does not pay now and never will
                c = T[i] * T[i] + T[j] * T[j] - 2 * T[i] * T[i] * N[i] + 2 * T[j] * T[j] * N[j]
                level = max(mu, Fraction(c, 2 * (T[j] - T[i])))
                if nxt is None or level < nxt[0]:
                    nxt = (level, i, j)
        if nxt is None or nxt[0] > mu_end:
            return best, arg, steps
        mu, i, j = nxt
        N[i] -= 1
        N[j] += 1
        steps += 1
        v = vx(T, N)
        if v < best:
            best, arg = v, list(N)


def pipelines_of(counts: Sequence[int], template_T: Sequence[int]) -> List[int]:
    """T of every pipeline of the plan `counts` (x_j pipelines of template j), template by template."""
    return [t for c, t in zip(counts, template_T) for _ in range(c)]


def plan_times(vectors: Sequence[Sequence[int]], template_T: Sequence[int], Q: int, solver=sweep):
    """For every count vector: (vx, time of the slowest pipeline under the distribution found), or
    None where Q microbatches cannot be distributed."""
    out = []
    for X in vectors:
        T = pipelines_of(X, template_T)
        res = solver(T, Q)
        if res[0] is None:
            out.append(None)
            continue
        N = res[1][0] if solver is exhaustive else res[1]
        out.append((res[0], max(n * t for n, t in zip(N, T))))
    return out


def best_plan(vectors: Sequence[Sequence[int]], template_T: Sequence[int], Q: int, solver=sweep) -> Optional[int]:
    """Index of the plan with the largest throughput (smallest slowest-pipeline time), the first of
    equals; None if no plan can take Q microbatches."""
    times = plan_times(vectors, template_T, Q, solver)
    best = None
    for i, r in enumerate(times):
        if r is not None and (best is None or r[1] < times[best][1]):
            best = i
    return best
