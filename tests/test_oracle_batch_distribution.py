"""Pins of the batch-distribution oracle (Section 4.2.2, Eq. 6): hand cases, a closed form,
the definition (exhaustive search) against the parametric method, invariances.  CPU only."""
import itertools
import random

from oracle import batch_distribution as BD


def test_hand_cases():
    # T = (2, 3), five microbatches: (1,4) -> times (2,12), (2,3) -> (4,9), (3,2) -> (6,6), (4,1) -> (8,3)
    assert [BD.vx([2, 3], N) for N in ([1, 4], [2, 3], [3, 2], [4, 1])] == [100, 25, 0, 25]
    assert BD.exhaustive([2, 3], 5) == (0, [[3, 2]])
    assert BD.sweep([2, 3], 5)[:2] == (0, [3, 2])
    # three equal pipelines, seven microbatches: one of them takes three; 3 (81+36+36) - 21^2 = 18
    v, arg = BD.exhaustive([3, 3, 3], 7)
    assert v == 18 and arg == [[2, 2, 3], [2, 3, 2], [3, 2, 2]]
    assert BD.sweep([3, 3, 3], 7)[0] == 18
    # twice as slow gets half as many
    assert BD.exhaustive([1, 2], 3) == (0, [[2, 1]])
    # fewer microbatches than pipelines: not distributable; exactly as many: one each
    assert BD.exhaustive([4, 5, 6], 2) == (None, []) and BD.sweep([4, 5, 6], 2)[0] is None
    assert BD.exhaustive([4, 5, 6], 3) == (3 * 77 - 225, [[1, 1, 1]]) and BD.sweep([4, 5, 6], 3)[:2] == (6, [1, 1, 1])


def test_equal_pipelines_closed_form():
    """x pipelines of equal T, Q = q x + r: r of them take q + 1, and x sum (a - mean)^2 = T^2 r (x - r)."""
    for T, x, Q in itertools.product([1, 7, 1000003], [1, 2, 3, 5, 8], range(1, 30)):
        if Q < x:
            continue
        q, r = divmod(Q, x)
        v, N, _ = BD.sweep([T] * x, Q)
        assert v == T * T * r * (x - r)
        assert sorted(N) == [q] * (x - r) + [q + 1] * r
        if x <= 3 or Q <= 12:
            assert BD.exhaustive([T] * x, Q)[0] == v


def test_definition_and_parametric_method_agree():
    rng = random.Random(6)
    ties = 0
    for case in range(2500):
        x = rng.randint(1, 5)
        Q = rng.randint(x, 14)
        T = [rng.choice([rng.randint(1, 50), rng.randint(1, 6), 7, rng.randint(10**8, 10**9)]) for _ in range(x)]
        v, arg = BD.exhaustive(T, Q)
        sv, sN, _ = BD.sweep(T, Q)
        assert sv == v and sN in arg, (T, Q)
        ties += len(arg) > 1
        assert sum(sN) == Q and min(sN) >= 1
    assert ties > 100  # the non-unique cases are part of the sample


def test_invariances():
    rng = random.Random(8)
    for case in range(300):
        x = rng.randint(2, 6)
        Q = rng.randint(x, 40)
        T = [rng.randint(1, 90) for _ in range(x)]
        v, N, _ = BD.sweep(T, Q)
        c = rng.randint(2, 9)
        assert BD.sweep([c * t for t in T], Q)[0] == c * c * v          # times scale, the variance with c^2
        perm = list(range(x))
        rng.shuffle(perm)
        assert BD.sweep([T[p] for p in perm], Q)[0] == v                 # the order of the pipelines is immaterial
        for i, j in itertools.permutations(range(x), 2):                 # no single exchange improves the result
            if N[i] >= 2:
                M = list(N)
                M[i] -= 1
                M[j] += 1
                assert BD.vx(T, M) >= v


def test_realistic_size_stays_near_the_continuous_level():
    """Sixteen pipelines, 512 microbatches, times of seconds in ns: every N_i T_i within one T_i of
    the level Q / sum(1 / T_i) that a fractional distribution would reach."""
    rng = random.Random(3)
    T = sorted(rng.randint(2 * 10**9, 9 * 10**9) for _ in range(16))
    v, N, steps = BD.sweep(T, 512)
    level = 512 / sum(1.0 / t for t in T)
    assert sum(N) == 512 and all(abs(n * t - level) <= t for n, t in zip(N, T))
    assert v == BD.vx(T, N) and steps > 0


def test_choice_between_plans_by_throughput():
    # two templates with T = 10 and 6; five microbatches; plans: two of the first, one of each, two of the second
    vectors, tt = [[2, 0], [1, 1], [0, 2]], [10, 6]
    assert BD.pipelines_of([1, 2], tt) == [10, 6, 6]
    # (10,10): 2+3 -> slowest 30; (10,6): N = (2,3) -> times (20,18), vx = 2*724 - 38^2 = 4; (6,6): 2+3 -> 18
    assert BD.plan_times(vectors, tt, 5) == [(100, 30), (4, 20), (36, 18)]
    assert BD.plan_times(vectors, tt, 5, solver=BD.exhaustive) == [(100, 30), (4, 20), (36, 18)]
    assert BD.best_plan(vectors, tt, 5) == 2
    assert BD.best_plan(vectors, tt, 1) is None
    assert BD.best_plan([[1, 0], [2, 0]], tt, 4) == 1   # 40 against 20
    assert BD.best_plan([[2, 0], [0, 2], [0, 2]], tt, 4) == 1  # the first of equals
