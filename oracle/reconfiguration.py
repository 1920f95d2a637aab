"""CPU oracle (test infrastructure only) of pipeline reinstantiation after node failures,
Section 5.1 (the three steps: simple reinstantiation, borrowing nodes, merging pipelines) and
Appendix B (a template exists for every merged pipeline).

State: the list of running pipelines, each a node count that is one of the template sizes
n0, n0+1, ..., n_hi (Section 4.1.1).  One *step* loses `burst` nodes, then repairs every
affected pipeline.  Plain Python, one trajectory at a time, in the paper's order of steps.

Where the paper leaves a choice open, this build reads it as follows:
  * which node fails: the caller's draw r (a 32-bit number) selects node
    floor(r * (nodes left) / 2^32), nodes counted pipeline after pipeline in list order;
  * training stops for good once fewer than (f+1) n0 nodes are left (Section 5, last sentence
    of its introduction); the step that gets there repairs nothing;
  * affected pipelines are repaired in list order;
  * a pipeline that still has n0 nodes or more is reinstantiated from the template of its new
    size (step 1);
  * a pipeline below n0 borrows one node at a time from the pipeline that has the most nodes
    among those above n0 (first in list order on ties) until it has n0 (step 2); the lenders
    are reinstantiated with fewer nodes;
  * when nobody can lend, it is merged with the smallest other pipeline (first in list order on
    ties), again and again until it has n0 nodes (step 3, Appendix B); a merged pipeline keeps
    the list position of the pipeline being repaired and the other one leaves the list.
Appendix B's claim is reported, not assumed: bit 0 of `violations` is set when a repaired
pipeline ends above n_hi (no template), bit 1 when fewer than f+1 pipelines are left after a
repair.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence

STOP_NONE, STOP_TOO_FEW_NODES, STOP_NO_PARTNER = 0, 1, 2


@dataclass
class StepRecord:
    reinstantiated: int = 0   # pipelines repaired by step 1 (lenders not counted)
    borrowed: int = 0         # nodes moved by step 2
    merges: int = 0           # pipelines absorbed by step 3
    alive: int = 0            # pipelines after the step
    stop: int = STOP_NONE


@dataclass
class Trajectory:
    steps: List[StepRecord] = field(default_factory=list)
    survived: int = 0         # steps repaired before training stopped
    sizes: List[int] = field(default_factory=list)  # per initial list position; 0 = gone
    violations: int = 0
    stop: int = STOP_NONE


def fail_node(sizes: List[Optional[int]], r: int) -> int:
    """Removes node floor(r * nodes left / 2^32) and returns the list position of its pipeline."""
    total = sum(s for s in sizes if s is not None)
    assert 0 <= r < 1 << 32
    r = (r * total) >> 32
    for i, s in enumerate(sizes):
        if s is None:
            continue
        if r < s:
            sizes[i] = s - 1
            return i
        r -= s
    raise AssertionError("unreachable")


def repair(sizes: List[Optional[int]], affected: Sequence[int], n0: int, n_hi: int, rec: StepRecord) -> int:
    """Section 5.1 on every affected pipeline, in list order.  `None` marks a list position whose
    pipeline was merged away.  Returns the violation bits of this repair (bit 0 only)."""
    viol = 0
    for i in sorted(set(affected)):
        if sizes[i] is None:
            continue
        if sizes[i] >= n0:                      # step 1: a template of this size exists
            rec.reinstantiated += 1
            continue
        while sizes[i] < n0:                    # step 2: borrow from whoever can yield
            lenders = [j for j, s in enumerate(sizes) if j != i and s is not None and s > n0]
            if not lenders:
                break
            j = max(lenders, key=lambda j: (sizes[j], -j))
            sizes[j] -= 1
            sizes[i] += 1
            rec.borrowed += 1
        while sizes[i] < n0:                    # step 3: merge
            others = [j for j, s in enumerate(sizes) if j != i and s is not None]
            if not others:
                rec.stop = STOP_NO_PARTNER
                return viol
            j = min(others, key=lambda j: (sizes[j], j))
            sizes[i] += sizes[j]
            sizes[j] = None
            rec.merges += 1
        if sizes[i] > n_hi:
            viol |= 1
    return viol


def simulate(sizes0: Sequence[int], n0: int, n_hi: int, f: int, draws: Sequence[Sequence[int]]) -> Trajectory:
    """One trajectory: draws[step][b] is the 32-bit draw of failure b of that step."""
    sizes: List[Optional[int]] = [int(s) for s in sizes0]
    tr = Trajectory()
    for step_draws in draws:
        rec = StepRecord()
        if tr.stop == STOP_NONE:
            affected = []
            for r in step_draws:
                if sum(s for s in sizes if s is not None) == 0:
                    break
                affected.append(fail_node(sizes, int(r)))
            if sum(s for s in sizes if s is not None) < (f + 1) * n0:
                rec.stop = STOP_TOO_FEW_NODES
            else:
                tr.violations |= repair(sizes, affected, n0, n_hi, rec)
                if rec.stop == STOP_NONE:
                    tr.survived += 1
                    if sum(1 for s in sizes if s is not None) < f + 1:
                        tr.violations |= 2
            tr.stop = rec.stop
        else:
            rec.stop = tr.stop
        rec.alive = sum(1 for s in sizes if s is not None)
        tr.steps.append(rec)
    tr.sizes = [0 if s is None else s for s in sizes]
    return tr
