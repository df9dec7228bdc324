"""Pins of the oracle's path-sampling estimator (Appendix C, Algorithm 1)."""
import itertools

import numpy as np

from oracle import rad_oracle as R


def layered_graph(rng, widths, fan):
    """Vertices level by level; every vertex of a level has `fan` distinct successors in later levels (the last
    level is the single output y).  Returns CSR arrays and per-level ranges."""
    starts = np.concatenate([[0], np.cumsum(widths)])
    n = int(starts[-1])
    succ_ptr, succ, partial = [0], [], []
    for l, w in enumerate(widths):
        for v in range(starts[l], starts[l + 1]):
            if l + 1 < len(widths):
                later = np.arange(starts[l + 1], n)
                pick = rng.choice(later, size=min(fan, len(later)), replace=False)
                succ += sorted(int(u) for u in pick)
                partial += list(rng.uniform(-1.5, 1.5, len(pick)))
            succ_ptr.append(len(succ))
    return np.array(succ_ptr), np.array(succ), np.array(partial), starts


def test_exact_adjoints_are_path_sums():
    # theta -> a, b -> y (a diamond) plus theta -> y: dy/dtheta = p_ta p_ay + p_tb p_by + p_ty
    succ_ptr = np.array([0, 3, 4, 5, 5]); succ = np.array([1, 2, 3, 3, 3])
    partial = np.array([2.0, -3.0, 0.5, 5.0, 7.0])
    adj = R.graph_exact_adjoints(succ_ptr, succ, partial, 3)
    assert adj.tolist() == [2 * 5 - 3 * 7 + 0.5, 5.0, 7.0, 1.0]


def test_expectation_over_every_outcome_is_the_exact_derivative():
    """k = 2 draws at every vertex of a small graph: the average of the estimate over all outcomes of all draws,
    enumerated (each outcome equally likely), is the exact derivative; vertices that were not reached
    contribute nothing and are reported unreached."""
    succ_ptr = np.array([0, 3, 5, 6, 6]); succ = np.array([1, 2, 3, 2, 3, 3])
    partial = np.array([2.0, -3.0, 0.5, 1.5, 5.0, 7.0])
    exact = R.graph_exact_adjoints(succ_ptr, succ, partial, 3)
    total, count, skipped = np.zeros(4), 0, 0
    for d0 in itertools.product(range(3), repeat=2):
        for d1 in itertools.product(range(2), repeat=2):
            for d2 in itertools.product(range(1), repeat=2):
                adj, reached = R.path_sample_adjoints(succ_ptr, succ, partial, 3, [0], 2, 0,
                                                      draws={0: d0, 1: d1, 2: d2})
                total += adj; count += 1
                skipped += int(not reached[1])
                assert np.all(adj[~reached] == 0.0)
    assert skipped > 0                                   # some outcomes never visit vertex 1
    np.testing.assert_allclose(total[0] / count, exact[0], rtol=1e-12)


def test_a_chain_is_exact_and_keys_pick_edges_by_the_replacement_rule():
    succ_ptr = np.arange(6); succ = np.arange(1, 6); partial = np.array([2.0, 3.0, -1.0, 0.5, 4.0])
    succ_ptr = np.concatenate([succ_ptr, [5]])
    adj, reached = R.path_sample_adjoints(succ_ptr, succ, partial, 5, [0], 3, seed=9)
    assert reached.all() and adj[0] == 2.0 * 3.0 * -1.0 * 0.5 * 4.0
    rng = np.random.default_rng(0)
    sp, su, pa, starts = layered_graph(rng, [1, 6, 1], 4)
    k, seed = 5, 123
    adj, reached = R.path_sample_adjoints(sp, su, pa, 7, [0], k, seed, stream_id=2)
    keys = R.element_keys(seed, 2, 0, 0, k)
    edges = [(int(kk) * 4) >> 32 for kk in keys]         # vertex 0 has 4 outgoing edges
    want = np.zeros(8, dtype=bool); want[0] = True; want[su[edges]] = True; want[7] = True
    assert np.array_equal(reached, want)


def test_mean_over_seeds_on_a_random_layered_graph():
    rng = np.random.default_rng(5)
    sp, su, pa, starts = layered_graph(rng, [3, 8, 8, 6, 1], 4)
    y = len(sp) - 2
    inputs = [0, 1, 2]
    exact = R.graph_exact_adjoints(sp, su, pa, y)
    S = 4000
    est = np.array([R.path_sample_adjoints(sp, su, pa, y, inputs, 3, s)[0][inputs] for s in range(S)])
    sem = est.std(axis=0) / np.sqrt(S)
    assert np.all(sem > 0) and np.all(np.abs(est.mean(axis=0) - exact[inputs]) < 4.5 * sem)
