"""Top-down memoised divide and conquer (Section 4.1.2), pure Python.

TEST INFRASTRUCTURE.  Second evaluation order of the same method: where the C
oracle fills tables bottom-up level by level, this one starts from the state
(S, 0, L, n*M) and recurses over (s, k, m) exactly as the "Divide" paragraph
describes, caching every intermediate result as the "memoization" paragraph
says.  It is only usable on small inputs.  Device sets are written here as
("G", g) for g GPUs inside a node and ("A", a) for a whole nodes.
"""
from __future__ import annotations

from typing import Dict, Optional, Tuple

FORBIDDEN = 1 << 62


class TopDown:
    def __init__(self, inp):
        self.inp = inp
        self.L, self.M, self.Nb = inp.L, inp.gpus_per_node, inp.microbatches
        self.cap = inp.mem_cap
        self.memo: Dict[tuple, Optional[tuple]] = {}

    def nb(self, S):
        return self.Nb if self.Nb > 0 else 4 * S

    # Eq. 4: a single stage on d GPUs of one node
    def stage(self, u, v, d):
        F, B = self.inp.fwd_ns, self.inp.bwd_ns
        t = 0
        for l in range(u, v):
            if F[l, d - 1] >= FORBIDDEN or B[l, d - 1] >= FORBIDDEN:
                return None
            t += int(F[l, d - 1]) + int(B[l, d - 1])
        bytes_ = sum(int(x) for x in self.inp.mem_bytes[u:v])
        if -((-bytes_) // d) > self.cap:
            return None
        if v < self.L:
            t += int(self.inp.boundary_ns[v - 1])
        return t

    def gpus(self, dev):
        return dev[1] if dev[0] == "G" else dev[1] * self.M

    def splits(self, dev):
        """Device pairs in increasing m."""
        if dev[0] == "A" and dev[1] >= 2:
            return [(m, ("A", m), ("A", dev[1] - m)) for m in range(1, dev[1])]
        g = self.gpus(dev)  # one node: GPUs are split
        return [(m, ("G", m), ("G", g - m)) for m in range(1, g)]

    def possible(self, S, dev):
        if self.Nb > 0 and S > self.Nb:
            return False
        if dev[0] == "G":
            return 1 <= dev[1] <= self.M - 1 and S <= dev[1]
        return dev[1] >= 1 and dev[1] <= S <= dev[1] * self.M

    def solve(self, S, u, v, dev) -> Optional[Tuple[int, int, int, int, tuple]]:
        """Returns (T1, T3, tmax, kstar, choice) or None."""
        key = (S, u, v, dev)
        if key in self.memo:
            return self.memo[key]
        res = None
        if not self.possible(S, dev) or v - u < S:
            res = None
        elif S == 1:
            t = self.stage(u, v, self.gpus(dev))
            res = None if t is None else (t, t, t, 0, (0, 0, 0))
        else:
            best = None
            for s in range(1, S):
                for k in range(u + s, v - (S - s) + 1):
                    for m, dl, dr in self.splits(dev):
                        a = self.solve(s, u, k, dl)
                        if a is None:
                            continue
                        b = self.solve(S - s, k, v, dr)
                        if b is None:
                            continue
                        T1 = a[0] + b[0]
                        if a[2] >= b[2]:
                            tmax, kstar, T3 = a[2], a[3], a[1] + b[0]
                        else:
                            tmax, kstar, T3 = b[2], s + b[3], b[1]
                        T = T1 + (self.nb(S) - S + kstar - 1) * tmax + T3
                        if best is None or T < best[0]:
                            best = (T, T1, T3, tmax, kstar, (s, k, m))
            res = None if best is None else best[1:]
        self.memo[key] = res
        return res

    def total(self, S, rec):
        return rec[0] + (self.nb(S) - S + rec[3] - 1) * rec[2] + rec[1]

    def stages(self, S, u, v, dev):
        if S == 1:
            return [(u, v, self.gpus(dev))]
        rec = self.solve(S, u, v, dev)
        s, k, m = rec[4]
        for mm, dl, dr in self.splits(dev):
            if mm == m:
                return self.stages(s, u, k, dl) + self.stages(S - s, k, v, dr)
        raise AssertionError

    def template(self, n):
        """Best (T, S, stages) over S in n..L for n nodes, or None."""
        best = None
        hi = min(self.L, n * self.M)
        if self.Nb > 0:
            hi = min(hi, self.Nb)
        for S in range(n, hi + 1):
            rec = self.solve(S, 0, self.L, ("A", n))
            if rec is None:
                continue
            T = self.total(S, rec)
            if best is None or T < best[0]:
                best = (T, S, rec)
        if best is None:
            return None
        T, S, rec = best
        return {"T": T, "S": S, "T1": rec[0], "T3": rec[1], "tmax": rec[2], "kstar": rec[3],
                "stages": self.stages(S, 0, self.L, ("A", n))}
