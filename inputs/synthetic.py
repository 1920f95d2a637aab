"""Seeded synthetic layer profiles shaped like GPT-style training workloads.

The planning method consumes, per layer l and per GPU count d = 1..M, a forward
and a backward time F_{l,d}, B_{l,d} (the profile of Eq. 4 in Section 4.1.2),
the memory a layer needs, and the cost of moving a stage boundary across the
network.  Real profiles are not available, so this module synthesises them
from a small portable generator.  Everything here is *data*: integer
nanoseconds and bytes.  None of the cost model or of the dynamic program lives
here, which is why the CPU oracle and the HIP path may both be fed from it.

Generator: SplitMix64, one stream per configuration (seed = configuration
seed).  Values are drawn layer by layer in the order  F, B-noise, state  (only
the fields that are random for that configuration consume draws).  For the
batched configuration each instance first draws L, then f, then its layers.

Units: MiB = 2**20 B, GiB = 2**30 B, GB/s = 10**9 B/s, times in ns.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

MiB = 1 << 20
GiB = 1 << 30
MASK64 = (1 << 64) - 1


class SplitMix64:
    """Portable 64-bit generator (Steele, Lea, Flood 2014 mixing function)."""

    def __init__(self, seed: int):
        self.state = seed & MASK64

    def next_u64(self) -> int:
        self.state = (self.state + 0x9E3779B97F4A7C15) & MASK64
        z = self.state
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & MASK64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & MASK64
        return z ^ (z >> 31)

    def uniform01(self) -> float:
        """Uniform double in [0, 1) with 53 random bits."""
        return (self.next_u64() >> 11) * (1.0 / (1 << 53))

    def randint(self, lo: int, hi: int) -> int:
        """Integer in [lo, hi] (inclusive; plain modulo reduction)."""
        return lo + self.next_u64() % (hi - lo + 1)

    def uniform(self, lo: float, hi: float) -> float:
        return lo + (hi - lo) * self.uniform01()

    def normal(self) -> float:
        """Standard normal by Box-Muller (one value per two uniforms)."""
        u1 = 1.0 - self.uniform01()  # (0, 1]
        u2 = self.uniform01()
        return math.sqrt(-2.0 * math.log(u1)) * math.cos(2.0 * math.pi * u2)

    def lognormal(self, median: float, sigma: float) -> float:
        return median * math.exp(sigma * self.normal())


def _ceil_div(a: int, b: int) -> int:
    return -((-a) // b)


@dataclass
class PlanInput:
    """One planning job: the profile arrays plus the scalar job arguments."""

    name: str
    fwd_ns: np.ndarray        # [L, M] int64, fwd_ns[l, d-1] = F_{l,d}
    bwd_ns: np.ndarray        # [L, M] int64, B_{l,d}
    mem_bytes: np.ndarray     # [L] int64, state + one microbatch of activations
    boundary_ns: np.ndarray   # [L] int64, time charged to a stage ending after layer l
    n_min: int
    n_max: int
    gpus_per_node: int
    microbatches: int
    mem_cap: int
    f: int
    meta: dict = field(default_factory=dict)

    @property
    def L(self) -> int:
        return int(self.mem_bytes.shape[0])


def make_profile(name: str, F1: List[int], B1: List[int], state: List[int],
                 act: List[int], boundary_bytes: List[int], link_Bps: int,
                 M: int, n_min: int, n_max: int, microbatches: int,
                 mem_cap: int, f: int, meta: Optional[dict] = None) -> PlanInput:
    """Expand single-GPU layer figures into the per-GPU-count tables.

    Rule of this build (the paper only says the times are profiled): running a
    layer on d GPUs of one node divides its time by d (rounded up) and adds a
    ring all-reduce of one boundary-sized tensor over an intra-node link that
    is 8x the inter-node link:
        F_{l,d} = ceil(F_{l,1} / d) + ceil(2 (d-1) bytes_l 1e9 / (d 8 link))
    and the same for B.  A stage that is not last pays one boundary-sized
    transfer forward and one back over the inter-node link:
        boundary_ns_l = 2 ceil(bytes_l 1e9 / link).
    """
    L = len(F1)
    fwd = np.zeros((L, M), dtype=np.int64)
    bwd = np.zeros((L, M), dtype=np.int64)
    for l in range(L):
        for d in range(1, M + 1):
            extra = 0
            if d > 1:
                extra = _ceil_div(2 * (d - 1) * boundary_bytes[l] * 10**9,
                                  d * 8 * link_Bps)
            fwd[l, d - 1] = _ceil_div(F1[l], d) + extra
            bwd[l, d - 1] = _ceil_div(B1[l], d) + extra
    mem = np.array([state[l] + act[l] for l in range(L)], dtype=np.int64)
    bnd = np.array([2 * _ceil_div(boundary_bytes[l] * 10**9, link_Bps)
                    for l in range(L)], dtype=np.int64)
    return PlanInput(name, fwd, bwd, mem, bnd, n_min, n_max, M, microbatches,
                     mem_cap, f, meta or {})


def _gpt_shaped(name, seed, layers, emb_mult, f_lo, f_hi, state_b, act_b,
                boundary_b, link, M, n_min, n_max, nb, cap, f):
    """`layers` transformer entries between an embedding entry and a head
    entry; the two extra entries cost emb_mult x a layer in time and memory."""
    rng = SplitMix64(seed)
    F1, B1, st, ac, bb = [], [], [], [], []
    for l in range(layers + 2):
        mult = emb_mult if (l == 0 or l == layers + 1) else 1
        fl = rng.randint(int(f_lo), int(f_hi)) * mult
        F1.append(fl)
        B1.append(2 * fl)
        st.append(state_b * mult)
        ac.append(act_b * mult)
        bb.append(boundary_b)
    return make_profile(name, F1, B1, st, ac, bb, link, M, n_min, n_max, nb,
                        cap, f, {"seed": seed, "layers": layers,
                                 "emb_mult": emb_mult})


def _config1() -> PlanInput:
    rng = SplitMix64(0)
    F1, B1, st = [], [], []
    for _ in range(12):
        fl = rng.randint(800_000, 1_200_000)
        bl = int(round(2 * fl * (1.0 + rng.uniform(-0.1, 0.1))))
        F1.append(fl)
        B1.append(bl)
        st.append(rng.randint(200 * MiB, 300 * MiB))
    return make_profile("cfg1_tiny", F1, B1, st, [40 * MiB] * 12, [8 * MiB] * 12,
                        25 * 10**9, 1, 1, 4, 8, 80 * GiB, 1, {"seed": 0})


def _config2() -> PlanInput:
    return _gpt_shaped("cfg2_gpt1p3b", 1, 24, 3, 2.0e6, 2.4e6, 300 * MiB,
                       96 * MiB, 16 * MiB, 25 * 10**9, 4, 2, 16, 32,
                       192 * GiB, 3)


def _config3() -> PlanInput:
    return _gpt_shaped("cfg3_gpt6p7b", 2, 32, 4, 6.0e6, 7.0e6,
                       int(1.6 * GiB), 256 * MiB, 32 * MiB, 25 * 10**9, 8, 4,
                       32, 64, 192 * GiB, 4)


def _config4() -> PlanInput:
    return _gpt_shaped("cfg4_gpt175b", 3, 96, 6, 4.5e7, 5.0e7, 30 * GiB,
                       3 * GiB // 2, 96 * MiB, 25 * 10**9, 8, 8, 64, 128,
                       192 * GiB, 8)


def _config5(count: int = 256) -> List[PlanInput]:
    rng = SplitMix64(7)
    out = []
    for idx in range(count):
        L = rng.randint(24, 128)
        f = rng.randint(1, 8)
        F1, B1, st = [], [], []
        for _ in range(L):
            fl = max(1, int(round(rng.lognormal(5.0e6, 0.5))))
            bl = max(1, int(round(fl * rng.uniform(1.8, 2.2))))
            F1.append(fl)
            B1.append(bl)
            st.append(max(1, int(round(rng.lognormal(float(GiB), 0.7)))))
        out.append(make_profile(f"cfg5_batch[{idx}]", F1, B1, st, [0] * L,
                                [32 * MiB] * L, 25 * 10**9, 8, 1, 32, 64,
                                192 * GiB, f, {"seed": 7, "instance": idx}))
    return out


_CONFIGS = {1: _config1, 2: _config2, 3: _config3, 4: _config4, 5: _config5}


def config_names():
    return {1: "tiny", 2: "gpt-1.3b-shaped", 3: "gpt-6.7b-shaped",
            4: "gpt-175b-shaped", 5: "batched-256"}


def config(idx: int):
    """Configuration 1-4: one PlanInput.  Configuration 5: a list of 256."""
    return _CONFIGS[idx]()


def random_small(seed: int, L: int, M: int, n_min: int, n_max: int, nb: int,
                 f: int = 1, tight_mem: bool = False, boundary: bool = True,
                 forbid_some_d: bool = False, t_lo: int = 1, t_hi: int = 50,
                 uniform_layers: bool = False) -> PlanInput:
    """Small random instance for tests (tiny integer times so that ties and
    every branch of the cost model occur often)."""
    rng = SplitMix64(0xC0FFEE ^ (seed * 0x9E3779B1))
    fwd = np.zeros((L, M), dtype=np.int64)
    bwd = np.zeros((L, M), dtype=np.int64)
    mem = np.zeros(L, dtype=np.int64)
    bnd = np.zeros(L, dtype=np.int64)
    f0, b0 = rng.randint(t_lo, t_hi), rng.randint(t_lo, t_hi)
    for l in range(L):
        fl = f0 if uniform_layers else rng.randint(t_lo, t_hi)
        bl = b0 if uniform_layers else rng.randint(t_lo, t_hi)
        for d in range(1, M + 1):
            sync = rng.randint(0, 3) if (d > 1 and not uniform_layers) else 0
            fwd[l, d - 1] = _ceil_div(fl, d) + sync
            bwd[l, d - 1] = _ceil_div(bl, d) + sync
        mem[l] = rng.randint(1, 10)
        bnd[l] = rng.randint(0, 5) if boundary else 0
    if forbid_some_d and M > 1:
        # forbid one GPU count for a couple of layers (2**62 marks "not allowed")
        for _ in range(2):
            l = rng.randint(0, L - 1)
            d = rng.randint(1, M)
            fwd[l, d - 1] = 1 << 62
            bwd[l, d - 1] = 1 << 62
    total = int(mem.sum())
    if tight_mem:
        cap = max(int(mem.max()), _ceil_div(total, max(1, (n_min + n_max) // 2 * M)) + rng.randint(0, 6))
    else:
        cap = total + 1
    return PlanInput(f"rand[{seed}]", fwd, bwd, mem, bnd, n_min, n_max, M, nb,
                     cap, f, {"seed": seed})
