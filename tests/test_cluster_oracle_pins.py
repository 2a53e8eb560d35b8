"""Pins of the operator-clustering oracle (Sec. 5.2, Eq. 6) against things other than itself."""
import numpy as np
import pytest

import oracle
from paper_2201_12023_amd import workloads as W
from tests.cluster_cases import INF64, enumerate_clusterings, layer_figures, load_example


def test_hand_worked_example():
    flop, src, dst, nb, cases = load_example()
    assert len(cases) == 6
    for L, delta, G, V, first in cases:
        g, v, f = oracle.cluster(flop, src, dst, nb, L, delta)
        assert (g, v, f) == (G, V, first), (L, delta)


@pytest.mark.parametrize("seed", range(40))
def test_first_component_is_the_optimum_over_all_clusterings(seed):
    rng = np.random.default_rng(seed)
    K = int(rng.integers(1, 11))
    g = W.random_op_graph(seed, K, int(rng.integers(0, 3 * K + 1)))
    for L in range(1, K + 1):
        delta = int(rng.choice([0, 100000, 500000, 2000000, 50000000]))
        every = enumerate_clusterings(g.flop, g.src, g.dst, g.nbytes, L, delta)
        G, V, first = oracle.cluster(g.flop, g.src, g.dst, g.nbytes, L, delta)
        if not every:
            assert G == INF64 and first == []
            continue
        best = min(e[0] for e in every)
        assert G == best
        # the clustering returned is one of the feasible ones and has the figures reported
        worst, sq, _ = layer_figures(g.flop, g.src, g.dst, g.nbytes, first)
        assert (worst, sq) == (G, V) and (worst, sq, first) in every
        # the tie-break never beats the best second component among optimal clusterings
        assert V >= min(e[1] for e in every if e[0] == best)


@pytest.mark.parametrize("seed", range(12))
def test_chain_graphs_second_component_is_optimal_too(seed):
    """Every operator feeds only the next one, with one size: every cut costs the same, so the
    choice is made by the FLOP spread alone and the recurrence is exact for it."""
    rng = np.random.default_rng(100 + seed)
    K = int(rng.integers(2, 11))
    flop = rng.integers(0, 12, size=K).astype(np.int32)
    src = np.arange(K - 1, dtype=np.int32)
    dst = src + 1
    nb = np.full(K - 1, 7, np.int64)
    for L in range(1, K + 1):
        every = enumerate_clusterings(flop, src, dst, nb, L, 1000000)
        G, V, first = oracle.cluster(flop, src, dst, nb, L, 1000000)
        if not every:
            assert G == INF64
            continue
        assert (G, V) == min((e[0], e[1]) for e in every)
        assert G == (0 if L == 1 else 7)


def test_closed_forms():
    g = W.random_op_graph(5, 9, 20)
    total = int(g.flop.sum())
    # one layer: nothing is received; the bound holds with delta = 0
    assert oracle.cluster(g.flop, g.src, g.dst, g.nbytes, 1, 0) == (0, total * total, [0, 9])
    # every operator alone (bound wide open): the largest in-degree weight
    indeg = np.zeros(9, np.int64)
    np.add.at(indeg, g.dst, g.nbytes)
    G, V, first = oracle.cluster(g.flop, g.src, g.dst, g.nbytes, 9, 10**9)
    assert G == int(indeg.max()) and first == list(range(10))
    assert V == int((g.flop.astype(np.int64) ** 2).sum())
    # more layers than operators: impossible
    assert oracle.cluster(g.flop, g.src, g.dst, g.nbytes, 10, 10**9)[0] == INF64
    # an operator heavier than the bound: impossible
    flop = np.asarray([1, 1, 50, 1, 1, 1], np.int32)
    e = np.arange(5, dtype=np.int32)
    assert oracle.cluster(flop, e, e + 1, np.ones(5, np.int64), 3, 0)[0] == INF64
    assert oracle.cluster(flop, e, e + 1, np.ones(5, np.int64), 3, 2000000)[0] == 1


@pytest.mark.parametrize("seed", range(6))
def test_invariants(seed):
    g = W.random_op_graph(200 + seed, 14, 30)
    L, delta = 4, 600000
    G, V, first = oracle.cluster(g.flop, g.src, g.dst, g.nbytes, L, delta)
    # scaling all byte counts scales G and leaves the clustering alone
    G3, V3, first3 = oracle.cluster(g.flop, g.src, g.dst, g.nbytes * 3, L, delta)
    assert (G3, V3, first3) == (3 * G if G != INF64 else INF64, V, first)
    # edge order does not matter
    perm = np.random.default_rng(seed).permutation(len(g.src))
    assert oracle.cluster(g.flop, g.src[perm], g.dst[perm], g.nbytes[perm], L, delta) == (G, V, first)
    # a looser FLOP bound never raises the first component
    G_loose = oracle.cluster(g.flop, g.src, g.dst, g.nbytes, L, 5 * delta)[0]
    assert G_loose <= G
    # an added edge never lowers it
    src = np.append(g.src, 0).astype(np.int32); dst = np.append(g.dst, 13).astype(np.int32)
    nb = np.append(g.nbytes, 9)
    assert oracle.cluster(g.flop, src, dst, nb, L, delta)[0] >= G
    # splitting an edge's bytes over two parallel edges changes nothing
    src2 = np.append(g.src, g.src[0]).astype(np.int32); dst2 = np.append(g.dst, g.dst[0]).astype(np.int32)
    nb2 = np.append(g.nbytes, g.nbytes[0] // 2); nb2[0] -= nb2[-1]
    assert oracle.cluster(g.flop, src2, dst2, nb2, L, delta) == (G, V, first)


def test_full_ties_go_to_the_earliest_cut():
    """Four unit-FLOP operators, edges 0->1 (5), 1->2 (7), 2->3 (5), 0->3 (100), two layers.
    Cut before op 1: layer 2 receives 0->1 and 0->3 = 105, FLOP 1|3, squares 10.
    Cut before op 2: receives 1->2 and 0->3 = 107.
    Cut before op 3: receives 2->3 and 0->3 = 105, FLOP 3|1, squares 10.
    The first and the third tie in both components; the recurrence keeps the lowest i."""
    G, V, first = oracle.cluster([1, 1, 1, 1], [0, 1, 2, 0], [1, 2, 3, 3], [5, 7, 5, 100], 2, 1000000)
    assert (G, V, first) == (105, 10, [0, 1, 4])


# ---------------------------------------------------------------- tie-break over whole clusterings


def test_exact_tie_break_worked_by_hand():
    """Four operators with FLOP 1, 4, 4, 3, edges 1->3 (2), 0->3 (2), 1->2 (1), three layers, no
    FLOP bound.  The three clusterings, from the definitions:
      {0} {1} {2,3}:  layer {2,3} receives 2 + 2 + 1 = 5;             squares 1 + 16 + 49 = 66
      {0} {1,2} {3}:  {1,2} receives nothing, {3} receives 2 + 2 = 4; squares 1 + 64 +  9 = 74
      {0,1} {2} {3}:  {2} receives 1, {3} receives 4;                 squares 25 + 16 + 9 = 50
    The smallest largest amount is 4, reached by the last two; of those the last has the more
    uniform layers.  The recurrence with its tie-break cell by cell settles G(3, 2) = 0 by
    {0} {1,2} (the other way to cut the first three operators costs 1) and so ends with 74."""
    args = ([1, 4, 4, 3], [1, 0, 1], [3, 3, 2], [2, 2, 1], 3, 10**9)
    assert oracle.cluster_exact(*args) == (4, 50, [0, 2, 3, 4])
    assert oracle.cluster(*args) == (4, 74, [0, 1, 3, 4])


@pytest.mark.parametrize("seed", range(40))
def test_exact_mode_is_the_lexicographic_optimum_over_all_clusterings(seed):
    """(largest amount received, sum of squared FLOP) is the smallest pair over every feasible
    clustering, and the clustering returned is, among those that reach it, the one whose last
    layer starts earliest, then whose last but one does, and so on (lowest i cell by cell on
    the way back)."""
    rng = np.random.default_rng(500 + seed)
    K = int(rng.integers(1, 11))
    g = W.random_op_graph(500 + seed, K, int(rng.integers(0, 3 * K + 1)),
                          flop_hi=int(rng.choice([2, 9])), bytes_hi=int(rng.choice([2, 6])))
    for L in range(1, K + 1):
        delta = int(rng.choice([0, 100000, 500000, 2000000, 50000000, 10**9]))
        every = enumerate_clusterings(g.flop, g.src, g.dst, g.nbytes, L, delta)
        G, V, first = oracle.cluster_exact(g.flop, g.src, g.dst, g.nbytes, L, delta)
        if not every:
            assert (G, V, first) == (INF64, 0, [])
            continue
        best = min((e[0], e[1]) for e in every)
        assert (G, V) == best
        optimal = [e[2] for e in every if (e[0], e[1]) == best]
        assert first == min(optimal, key=lambda f: tuple(reversed(f[1:-1])))
        Gc, Vc, _ = oracle.cluster(g.flop, g.src, g.dst, g.nbytes, L, delta)
        assert Gc == G and Vc >= V                 # the cell-by-cell rule: same G, never better


def test_exact_mode_differs_from_the_cell_by_cell_rule_somewhere():
    n = 0
    for seed in range(60):
        g = W.random_op_graph(900 + seed, 9, 20, flop_hi=5, bytes_hi=3)
        for L in (3, 4, 5):
            a = oracle.cluster(g.flop, g.src, g.dst, g.nbytes, L, 10**9)
            b = oracle.cluster_exact(g.flop, g.src, g.dst, g.nbytes, L, 10**9)
            assert a[0] == b[0] and a[1] >= b[1]
            n += a[1] > b[1]
    assert n >= 3


def test_exact_mode_closed_forms_and_chains():
    g = W.random_op_graph(5, 9, 20)
    total = int(g.flop.sum())
    assert oracle.cluster_exact(g.flop, g.src, g.dst, g.nbytes, 1, 0) == (0, total * total, [0, 9])
    assert oracle.cluster_exact(g.flop, g.src, g.dst, g.nbytes, 10, 10**9)[0] == INF64
    G, V, first = oracle.cluster_exact(g.flop, g.src, g.dst, g.nbytes, 9, 10**9)
    assert first == list(range(10)) and V == int((g.flop.astype(np.int64) ** 2).sum())
    # chain graphs: every cut costs the same, the two rules agree in (G, V)
    for seed in range(8):
        rng = np.random.default_rng(300 + seed)
        K = int(rng.integers(2, 11))
        flop = rng.integers(0, 12, size=K).astype(np.int32)
        src = np.arange(K - 1, dtype=np.int32)
        nb = np.full(K - 1, 7, np.int64)
        for L in range(1, K + 1):
            a = oracle.cluster(flop, src, src + 1, nb, L, 1000000)
            b = oracle.cluster_exact(flop, src, src + 1, nb, L, 1000000)
            assert a[:2] == b[:2]
