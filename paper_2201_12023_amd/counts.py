"""Work-unit counters for the stage-slicing DP (host-side bookkeeping for the benchmark).

A *cell* is one F(s, k, d) of Eq. 3; a *cell-update* is one (last layer i, shape q) term
of one cell.  ``n_dense`` counts what the loop nest of Alg. 1 visits (s = 1..K, every
i >= k, every shape with a_q <= d); ``n_struct`` counts only the terms whose F(s-1, ...)
operand is not infinite by index structure alone (s = 1: i = K and a_q = d; s > 1: at
least s - 1 layers and s - 1 devices remain after the stage).  Both are per candidate.
"""
from __future__ import annotations


def work_counts(K: int, D: int, sizes) -> dict:
    sizes = [int(a) for a in sizes]
    cells = K * K * D
    n_dense = 0
    for d in range(1, D + 1):
        nq = sum(1 for a in sizes if a <= d)
        n_dense += nq
    n_dense *= K * (K * (K + 1) // 2)
    n_struct = 0
    for s in range(1, K + 1):
        if s == 1:
            n_struct += K * sum(1 for a in sizes if a <= D)
            continue
        n = K - s + 1                      # last layers i with K - i >= s - 1
        if n <= 0:
            break
        pairs = n * (n + 1) // 2           # (k, i) with k <= i <= n
        for a in sizes:
            nd = D - (a + s - 1) + 1
            if nd > 0:
                n_struct += pairs * nd
    return dict(cells=cells, n_dense=n_dense, n_struct=n_struct)
