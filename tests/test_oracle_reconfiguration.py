"""Pins of the reconfiguration oracle (Section 5.1, Appendix B): the three cases the paper
draws, closed forms and invariants.  CPU only."""
import itertools

import numpy as np

import inputs
from oracle import reconfiguration as R


def draw_for(node, total):
    """The smallest draw that selects `node` out of `total` nodes."""
    return -(-(node << 32) // total)


def one_failure_in(sizes, which):
    """A draw that makes the first node of pipeline `which` fail."""
    return draw_for(sum(sizes[:which]), sum(sizes))


def test_the_three_cases_of_the_reinstantiation_figure():
    # templates for 2, 3 and 4 nodes (the sizes of the paper's examples), f = 1
    # (a) a node of a 4-node pipeline fails; a 3-node template exists: plain reinstantiation
    tr = R.simulate([4, 2], 2, 4, 1, [[one_failure_in([4, 2], 0)]])
    assert tr.sizes == [3, 2] and (tr.steps[0].reinstantiated, tr.steps[0].borrowed, tr.steps[0].merges) == (1, 0, 0)
    # (b) a node of a 2-node pipeline fails; there is no 1-node template: it takes a node from the
    #     other pipeline and stays a 2-node pipeline, the lender shrinks
    tr = R.simulate([2, 3, 2], 2, 4, 1, [[one_failure_in([2, 3, 2], 0)]])
    assert tr.sizes == [2, 2, 2] and (tr.steps[0].reinstantiated, tr.steps[0].borrowed, tr.steps[0].merges) == (0, 1, 0)
    # (c) nobody can yield a node: the pipeline is merged with another one
    tr = R.simulate([2, 2, 2], 2, 4, 1, [[one_failure_in([2, 2, 2], 1)]])
    assert tr.sizes == [0, 3, 2] and (tr.steps[0].reinstantiated, tr.steps[0].borrowed, tr.steps[0].merges) == (0, 0, 1)
    assert tr.steps[0].alive == 2 and tr.violations == 0 and tr.survived == 1


def test_node_selection_counts_nodes_pipeline_after_pipeline():
    """Ten nodes in pipelines of 3, 3 and 4: node = floor(draw * 10 / 2^32); draws worked by hand
    (1288490189 = ceil(3 * 2^32 / 10), 2576980378 = ceil(6 * 2^32 / 10))."""
    for r, want in [(0, [2, 3, 4]), (1288490188, [2, 3, 4]), (1288490189, [3, 2, 4]), (1 << 31, [3, 2, 4]),
                    (2576980377, [3, 2, 4]), (2576980378, [3, 3, 3]), (2**32 - 1, [3, 3, 3])]:
        sizes = [3, 3, 4]
        i = R.fail_node(sizes, r)
        assert sizes == want and sizes[i] == want[i], (r, sizes)
    sizes = [3, None, 4]
    assert R.fail_node(sizes, draw_for(3, 7)) == 2 and sizes == [3, None, 3]
    assert R.fail_node(sizes, draw_for(3, 6) - 1) == 0 and sizes == [2, None, 3]


def test_training_survives_exactly_down_to_f_plus_one_smallest_pipelines():
    """One failure per step: with the node specification of Section 4.1.1 (consecutive sizes up to
    N - f n0 and more sizes than n0 - 1) every trajectory repairs exactly N - (f+1) n0 failures,
    keeps the node count, keeps every pipeline on a template size and keeps f+1 pipelines
    (Appendix B), whatever nodes fail."""
    checked = 0
    for n0, f, extra in itertools.product([1, 2, 3, 5], [0, 1, 2, 3], [0, 1, 4, 9]):
        N = (f + 1) * n0 + max(extra, n0 - 1 if f == 0 else 0) + n0   # room for p > n0 - 1 sizes
        n_hi = N - f * n0
        if n_hi - n0 + 1 <= n0 - 1:
            continue
        for seed in range(6):
            sizes0 = inputs.starting_pipelines(seed, n0, n_hi, N, f)
            steps = N
            draws = inputs.failure_draws(100 + seed, steps, 1, 1)[:, :, 0]
            tr = R.simulate(sizes0, n0, n_hi, f, draws)
            assert tr.survived == N - (f + 1) * n0, (n0, f, N, list(sizes0))
            assert tr.violations == 0
            assert tr.stop == R.STOP_TOO_FEW_NODES
            assert sum(tr.sizes) == (f + 1) * n0 - 1
            # replay step by step: after every repaired step the state is a valid instantiation
            for k in range(1, tr.survived + 1):
                part = R.simulate(sizes0, n0, n_hi, f, draws[:k])
                alive = [s for s in part.sizes if s]
                assert sum(alive) == N - k and all(n0 <= s <= n_hi for s in alive) and len(alive) >= f + 1
                assert part.steps[-1].alive == len(alive)
            checked += 1
    assert checked > 200


def test_merging_happens_only_when_nobody_can_lend_and_lands_below_twice_n0():
    """Appendix B: a merge of pipelines that could not borrow ends with n0 <= size < 2 n0."""
    rng = np.random.Generator(np.random.PCG64(5))
    merges = 0
    for case in range(300):
        n0 = int(rng.integers(2, 7))
        f = int(rng.integers(0, 4))
        c = f + 1 + int(rng.integers(1, 5))
        sizes0 = [n0] * c                      # nobody can lend
        k = int(rng.integers(1, n0))           # lose k nodes of one pipeline in one burst
        which = int(rng.integers(0, c))
        draws = [[draw_for(which * n0, c * n0 - b) for b in range(k)]]
        tr = R.simulate(sizes0, n0, 2 * n0 - 1, f, draws)
        assert tr.steps[0].merges == 1 and tr.steps[0].borrowed == 0
        assert tr.sizes[which] == 2 * n0 - k and sorted(tr.sizes)[0] == 0 and tr.violations == 0
        merges += 1
    assert merges == 300


def test_bursts_conserve_nodes_and_keep_template_sizes():
    for seed in range(40):
        rng = np.random.Generator(np.random.PCG64(seed))
        n0, f = int(rng.integers(2, 6)), int(rng.integers(0, 4))
        N = (f + 1) * n0 + int(rng.integers(n0, 4 * n0))
        n_hi = N - f * n0
        burst = int(rng.integers(2, 5))
        sizes0 = inputs.starting_pipelines(seed, n0, n_hi, N, f)
        draws = inputs.failure_draws(seed, N, burst, 1)[:, :, 0]
        tr = R.simulate(sizes0, n0, n_hi, f, draws)
        lost = burst * tr.survived
        alive = [s for s in tr.sizes]
        assert tr.stop == R.STOP_TOO_FEW_NODES
        assert N - lost - burst <= sum(alive) < (f + 1) * n0
        for k in range(1, tr.survived + 1):
            part = R.simulate(sizes0, n0, n_hi, f, draws[:k])
            live = [s for s in part.sizes if s]
            assert sum(live) == N - burst * k
            assert all(s >= n0 for s in live)
            if not part.violations & 1:
                assert all(s <= n_hi for s in live)


def test_the_choices_the_paper_leaves_open_follow_the_stated_reading():
    """Worked by hand from the reading in the oracle's header."""
    # the lender is the largest pipeline above n0, the first of equals
    assert R.simulate([2, 3, 4], 2, 4, 1, [[0]]).sizes == [2, 3, 3]
    assert R.simulate([2, 3, 3], 2, 4, 1, [[0]]).sizes == [2, 2, 3]
    # two nodes short ([1, 3, 4], n0 = 3): the 4 lends one, then nobody can: merge with the first 3
    tr = R.simulate([3, 3, 4], 3, 5, 0, [[0, 0]])
    assert tr.sizes == [5, 0, 3] and (tr.steps[0].borrowed, tr.steps[0].merges) == (1, 1)
    # [1, 3, 2] after the burst: the merge partner is the smallest other pipeline, not the first
    tr = R.simulate([3, 3, 3], 3, 5, 0, [[0, 0, draw_for(6, 7)]])
    assert tr.sizes == [3, 3, 0] and (tr.steps[0].borrowed, tr.steps[0].merges) == (0, 1)
    # [2, 2, 2, 3] after the burst, f = 2: the first pipeline absorbs the second (4 nodes) and then
    # lends a node to the third: three pipelines of three nodes are left
    tr = R.simulate([3, 3, 3, 3], 3, 5, 2, [[0, draw_for(3, 11), draw_for(6, 10)]])
    assert tr.sizes == [3, 0, 3, 3] and (tr.steps[0].borrowed, tr.steps[0].merges, tr.steps[0].alive) == (1, 1, 3)
    assert tr.violations == 0
    # fewer than (f+1) n0 nodes: training stops, nothing is repaired, later steps change nothing
    tr = R.simulate([2, 2], 2, 3, 1, [[0], [0]])
    assert tr.sizes == [1, 2] and tr.survived == 0 and [r.stop for r in tr.steps] == [1, 1]


def test_counts_and_violation_flags_on_hand_cases():
    # a pipeline that lands exactly on n0 is a plain reinstantiation
    tr = R.simulate([3, 2], 2, 4, 0, [[0]])
    assert tr.sizes == [2, 2] and (tr.steps[0].reinstantiated, tr.steps[0].borrowed, tr.steps[0].merges) == (1, 0, 0)
    # two sizes only (3 and 4) although n0 - 1 = 2 would need more than two (Section 4.1.1): the merge
    # of a 2-node rest with a 3-node pipeline has 5 nodes and no template; with a 5-node template it has
    assert R.simulate([3, 3], 3, 4, 0, [[0]]).violations == 1
    assert R.simulate([3, 3], 3, 4, 0, [[0]]).sizes == [5, 0]
    assert R.simulate([3, 3], 3, 5, 0, [[0]]).violations == 0
    # a start with fewer than f+1 pipelines is reported once a step has been repaired
    tr = R.simulate([4, 4], 2, 4, 2, [[0]])
    assert tr.sizes == [3, 4] and tr.violations == 2 and tr.survived == 1
    assert R.simulate([4, 4], 2, 4, 1, [[0]]).violations == 0
