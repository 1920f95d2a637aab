"""Batch distribution (Section 4.2.2, Eq. 6) and plan choice through the C ABI against the CPU oracle.
The minimum of Eq. 6 is unique and compared exactly (128-bit integers); the distribution that
reaches it is not, so it is checked for validity: it uses Q microbatches, at least one per pipeline,
and has exactly the minimal variance and the reported slowest time."""
import random

import numpy as np
import pytest

import inputs
from oracle import batch_distribution as BD

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import torch
    import paper_2309_08125_amd as pkg

    assert torch.cuda.is_available()
    pkg.load()
    return pkg


def distribution_of(X, base, extra):
    N = []
    for c, b, e in zip(X, base, extra):
        assert (c > 0) or (b == 0 and e == 0)
        assert e <= c
        N += [int(b) + 1] * int(e) + [int(b)] * (int(c) - int(e))
    return N


def compare(P, vectors, template_T, Q, exhaustive):
    st, vx, slow, base, extra = P.Distributor(vectors, len(vectors), template_T, Q).solve()
    for i, X in enumerate(vectors):
        T = BD.pipelines_of(X, template_T)
        if not T:
            assert st[i] == P.OOB_DIST_NO_PIPELINE
            continue
        if len(T) > Q:
            assert st[i] == P.OOB_DIST_TOO_FEW_MICROBATCHES and vx[i] == 0 and slow[i] == 0 and not base[i].any()
            continue
        assert st[i] == P.OOB_DIST_OK, (X, st[i])
        N = distribution_of(X, base[i], extra[i])
        assert sum(N) == Q and min(N) >= 1, (X, N)
        want = BD.exhaustive(T, Q)[0] if exhaustive else BD.sweep(T, Q)[0]
        assert vx[i] == want == BD.vx(T, N), (X, template_T, Q, N)
        assert slow[i] == max(n * t for n, t in zip(N, T))
    return st, vx, slow


def test_hand_cases(P):
    # templates with T = 10 and 6, five microbatches (worked in the oracle's pins): (10,10) -> 2+3, slowest 30;
    # (10,6) -> N = (2,3), x sum of squares 4, slowest 20; (6,6) -> slowest 18
    d = P.Distributor([[2, 0], [1, 1], [0, 2]], 3, [10, 6], 5)
    st, vx, slow, base, extra = d.solve()
    assert st.tolist() == [0, 0, 0] and vx == [100, 4, 36] and slow.tolist() == [30, 20, 18]
    assert base.tolist() == [[2, 0], [2, 3], [0, 2]] and extra.tolist() == [[1, 0], [0, 0], [0, 1]]
    assert d.choose([0, 3]).tolist() == [2]
    assert d.choose([0, 1, 2, 3, 3]).tolist() == [0, 1, 2, -1]
    # T = (2, 3), five microbatches: N = (3, 2), all pipelines take 6
    st, vx, slow, base, extra = P.Distributor([[1, 1]], 1, [2, 3], 5).solve()
    assert (vx, slow.tolist(), base.tolist(), extra.tolist()) == ([0], [6], [[3, 2]], [[0, 0]])


def test_small_plans_against_the_definition(P):
    """Every plan against exhaustive search: few pipelines, few microbatches, equal and very
    different times, plans that cannot be distributed, several workgroups and a ragged last one."""
    rng = random.Random(4)
    plans = 0
    for case in range(120):
        p = rng.randint(1, 5)
        tT = [rng.choice([rng.randint(1, 60), rng.randint(10**8, 10**9), 7]) for _ in range(p)]
        Q = rng.randint(1, 13)
        vecs = [[rng.choice([0, 0, 1, 1, 2, 3]) for _ in range(p)] for _ in range(rng.randint(1, 150))]
        vecs = [v for v in vecs if sum(v) <= 6]
        if vecs:
            compare(P, vecs, tT, Q, exhaustive=True)
            plans += len(vecs)
    assert plans > 3000


def test_realistic_plans_against_the_parametric_oracle(P):
    """Up to 16 pipelines, up to 512 microbatches, times of seconds in ns (up to the library's limit)."""
    rng = random.Random(5)
    for case in range(25):
        p = rng.randint(2, 24)
        tT = sorted(rng.randint(2 * 10**9, (1 << 35)) for _ in range(p))
        Q = rng.choice([32, 100, 256, 512])
        vecs = []
        for _ in range(24):
            v = [0] * p
            for _ in range(rng.randint(1, 16)):
                v[rng.randrange(p)] += 1
            vecs.append(v)
        print("case", case, p, Q, flush=True)
        compare(P, vecs, tT, Q, exhaustive=False)


def test_templates_of_nearly_equal_time(P):
    """Times that differ by a few ns in 10^10: the levels of the exchanges then cancel to a small
    part of their terms: only exact integer comparisons order them correctly."""
    rng = random.Random(9)
    for case in range(30):
        base = rng.randint(10**9, 3 * 10**10)
        tT = sorted(set(base + rng.randint(0, 6) for _ in range(rng.randint(2, 8))))
        Q = rng.choice([20, 64, 200])
        vecs = [[rng.choice([0, 1, 1, 2]) for _ in range(len(tT))] for _ in range(40)]
        vecs = [v for v in vecs if 0 < sum(v) <= Q]
        compare(P, vecs, tT, Q, exhaustive=False)


def test_status_codes_and_limits(P):
    tT = list(range(100, 120))
    x17 = [1] * 17 + [0] * 3          # seventeen templates in one plan
    x16 = [1] * 16 + [0] * 4
    st, vx, slow, base, extra = P.Distributor([x17, x16, [0] * 20], 3, tT, 40).solve()
    assert st.tolist() == [P.OOB_DIST_TOO_MANY_TEMPLATES, P.OOB_DIST_OK, P.OOB_DIST_NO_PIPELINE]
    assert vx[0] == 0 and not base[0].any() and vx[1] == BD.sweep(BD.pipelines_of(x16, tT), 40)[0]
    st = P.Distributor([[1, 1, 0], [1, 0, 1], [1, 0, 0]], 3, [5, 0, (1 << 35) + 1], 9).solve()[0]
    assert st.tolist() == [P.OOB_DIST_BAD_TIME, P.OOB_DIST_BAD_TIME, P.OOB_DIST_OK]
    # the largest time and the largest Q the library takes, two pipelines
    big = 1 << 35
    st, vx, slow, base, extra = P.Distributor([[1, 1]], 1, [big, big - 1], 65535).solve()
    assert st.tolist() == [0] and vx[0] == BD.sweep([big, big - 1], 65535)[0]
    fake = 0x10000
    assert P.oob_dist_solve(0, 1, 1, 1, fake, 1, fake, fake, 0, 0, fake, 0) == P.OOB_EINVAL
    assert P.oob_dist_solve(fake, 2, 1, 1, fake, 1, fake, fake, 0, 0, fake, 0) == P.OOB_EINVAL   # capacity < count
    assert P.oob_dist_solve(fake, 1, 1, 1, fake, 0, fake, fake, 0, 0, fake, 0) == P.OOB_EINVAL   # Q
    assert P.oob_dist_solve(fake, 1, 1, 1, fake, 1, fake, fake, fake, 0, fake, 0) == P.OOB_EINVAL  # base without extra
    assert P.oob_dist_solve(fake, 0, 0, 1, fake, 1, fake, fake, 0, 0, fake, 0) == P.OOB_OK        # nothing to do


def test_choice_of_the_plan_against_the_oracle(P):
    """Groups of plans as the enumeration produces them (one group per cluster size); cases in which
    every minimiser of a plan has the same slowest time, so that the choice is unique."""
    rng = random.Random(7)
    checked = 0
    for case in range(40):
        sizes = sorted(rng.sample(range(2, 9), rng.randint(2, 4)))
        tT = [rng.randint(20, 60) * 100 // n for n in sizes]
        Q = rng.randint(6, 12)
        from oracle import instantiation

        off, vecs = instantiation.instantiations_range(sizes, 6, 16, 1)
        vecs = [list(map(int, v)) for v in vecs]
        unique = all(len({max(n * t for n, t in zip(N, BD.pipelines_of(X, tT))) for N in BD.exhaustive(BD.pipelines_of(X, tT), Q)[1]}) <= 1
                     for X in vecs)
        if not unique or not vecs:
            continue
        d = P.Distributor(vecs, len(vecs), tT, Q)
        d.solve()
        best = d.choose(off)
        for g in range(len(off) - 1):
            want = BD.best_plan(vecs[off[g]:off[g + 1]], tT, Q, solver=BD.exhaustive)
            assert best[g] == (-1 if want is None else off[g] + want), (sizes, tT, Q, g)
        checked += 1
    assert checked >= 15


def test_headline_node_specification_at_full_size(P):
    """All 1 343 380 plans of the headline workload's node specification (templates for 8..64 nodes,
    f = 8, 72..128 nodes), the planner's own T1 per template as the time per microbatch, 512
    microbatches, as bench.py runs it: sampled plans against the oracle, all of them against what
    holds for any correct output."""
    import torch

    inp = inputs.config(4)
    planner = P.Planner(inp.L, inp.n_max, inp.gpus_per_node)
    res = planner.plan(inp)
    planner.close()
    n0, n_hi, p, N = (int(v) for v in res["cover_hdr"][:4])
    tT = [int(v) for v in res["T1"][n0 - inp.n_min: n0 - inp.n_min + p]]
    inst = P.Instantiator(None, (inp.f + 1) * n0, N, inp.f, n0=n0, p=p)
    off, st = inst.count()
    total = int(off[-1])
    x = torch.empty((p, total), dtype=torch.int16, device="cuda")
    inst.enqueue(x, total)
    Q = 512
    d = P.Distributor(x, total, tT, Q)
    st, vx, slow, base, extra = d.solve()
    assert total == 1343380 and (st == P.OOB_DIST_OK).all()
    X = x.cpu().numpy().view("uint16").T
    pipes = X.sum(axis=1)
    assert (((base.astype(np.int64) * X) + extra).sum(axis=1) == Q).all()      # every microbatch is handed out
    assert (base[X > 0] >= 1).all() and (extra <= X).all()
    times = (base.astype(np.int64) + (extra > 0)) * np.asarray(tT, dtype=np.int64)[None, :]
    assert (times.max(axis=1) == slow).all()
    assert (slow * pipes >= Q * min(tT)).all()
    rng = np.random.Generator(np.random.PCG64(2))
    for i in rng.integers(0, total, size=120).tolist() + [0, total - 1]:
        T = BD.pipelines_of(X[i].tolist(), tT)
        Nd = distribution_of(X[i].tolist(), base[i], extra[i])
        assert vx[i] == BD.sweep(T, Q)[0] == BD.vx(T, Nd), i
    best = d.choose(off)
    for g in range(len(off) - 1):
        seg = slow[off[g]:off[g + 1]]
        assert best[g] == off[g] + int(np.argmin(seg))
