"""Seeded synthetic failure sequences and starting pipeline sets for the reconfiguration
simulator.  Data only: which node a draw selects and what happens then is the method's business
and lives in the oracle and in the HIP path, separately."""
from __future__ import annotations

import numpy as np


def failure_draws(seed: int, steps: int, burst: int, trajectories: int) -> np.ndarray:
    """uint32 draws, shape (steps, burst, trajectories): draw [s, b, t] selects the node that
    fails as failure b of step s in trajectory t."""
    rng = np.random.Generator(np.random.PCG64(seed))
    return rng.integers(0, 1 << 32, size=(steps, burst, trajectories), dtype=np.uint64).astype(np.uint32)


def starting_pipelines(seed: int, n0: int, n_hi: int, N: int, f: int) -> np.ndarray:
    """Some set of at least f+1 pipelines with sizes in [n0, n_hi] that uses exactly N nodes."""
    assert N >= (f + 1) * n0 and n0 <= n_hi
    rng = np.random.Generator(np.random.PCG64(seed))
    sizes = [n0] * (f + 1)
    left = N - (f + 1) * n0
    while left > 0:
        room = [i for i, s in enumerate(sizes) if s < n_hi]
        if left >= n0 and (not room or rng.random() < 0.35):
            sizes.append(n0)
            left -= n0
            continue
        assert room, "N does not fit these sizes"
        sizes[room[int(rng.integers(0, len(room)))]] += 1
        left -= 1
    order = rng.permutation(len(sizes))
    return np.asarray(sizes, dtype=np.int32)[order]
