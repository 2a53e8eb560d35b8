"""Reader of the hand-worked clustering example and an enumeration of every clustering."""
import itertools
import os

import numpy as np

INF64 = 2**63 - 1
_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "cluster_example.txt")


def load_example():
    """Returns (flop, src, dst, nbytes, cases); a case is (L, delta_ppm, G, V, first_op)."""
    flop, edges, cases = [], [], []
    for line in open(_PATH):
        line = line.split("#")[0].split()
        if not line:
            continue
        if line[0] == "flop":
            flop = [int(x) for x in line[1:]]
        elif line[0] == "edge":
            edges.append([int(x) for x in line[1:]])
        elif line[0] == "case":
            v = [INF64 if x == "INF" else int(x) for x in line[1:]]
            cases.append((v[0], v[1], v[2], v[3], v[4:]))
    e = np.asarray(edges, np.int64).reshape(-1, 3)
    return (np.asarray(flop, np.int32), e[:, 0].astype(np.int32), e[:, 1].astype(np.int32),
            e[:, 2].astype(np.int64), cases)


def layer_figures(flop, src, dst, nbytes, first_op):
    """(largest amount of data a layer receives from earlier operators, sum of squared FLOP,
    largest per-layer FLOP) of a given clustering, from the definitions."""
    worst, sq, fmax = 0, 0, 0
    for a, b in zip(first_op[:-1], first_op[1:]):
        assert a < b
        recv = sum(int(w) for u, v, w in zip(src, dst, nbytes) if u < a <= v < b)
        f = int(np.sum(flop[a:b], dtype=np.int64))
        worst, sq, fmax = max(worst, recv), sq + f * f, max(fmax, f)
    return worst, sq, fmax


def enumerate_clusterings(flop, src, dst, nbytes, L, delta_ppm):
    """Every way to cut K operators into L non-empty consecutive layers that keeps each
    layer's FLOP within the bound: list of (largest received, sum of squares, first_op)."""
    K = len(flop)
    total = int(np.sum(flop, dtype=np.int64))
    out = []
    for cuts in itertools.combinations(range(1, K), L - 1):
        first = [0, *cuts, K]
        worst, sq, fmax = layer_figures(flop, src, dst, nbytes, first)
        if fmax * L * 1000000 <= (1000000 + delta_ppm) * total:
            out.append((worst, sq, first))
    return out
