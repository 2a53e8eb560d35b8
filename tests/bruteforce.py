"""Brute-force statement of Eq. 2 (Sec. 5.1), independent of the oracle's recurrence.

Enumerates every way to cut layers 0..K-1 into contiguous stages and to give each
stage one of the allowed submesh shapes so that the device counts add up to N*M
exactly (the covering condition of Sec. 5.2), looks each stage's latency up in the
table (third index: number of stages from this one to the last, inclusive) and
evaluates  sum t + (B - 1) * max t  directly.  Pure Python, small K only.
"""
from __future__ import annotations

INF32 = 2**31 - 1


def enumerate_plans(table, K, D, sizes):
    """Yield (stages, lat) with stages = [(first, last, q), ...] in pipeline order and
    lat = the per-stage latencies, for every plan whose entries are all finite."""
    S = len(sizes)
    out = []

    def rec(k, d, acc):
        if k == K:
            if d == 0 and acc:
                out.append(list(acc))
            return
        if d <= 0:
            return
        for i in range(k, K):
            for q in range(S):
                if sizes[q] <= d:
                    acc.append((k, i, q))
                    rec(i + 1, d - sizes[q], acc)
                    acc.pop()

    rec(0, D, [])
    for stages in out:
        n = len(stages)
        lat = []
        ok = True
        for p, (k, i, q) in enumerate(stages):
            s = n - p                      # stages from this one to the last, inclusive
            t = int(table[s - 1][k][i][q])
            if t == INF32:
                ok = False
                break
            lat.append(t)
        if ok:
            yield stages, lat


def solve(table, K, D, sizes, B):
    """Returns dict with: T_star, t_max, stages (the plan selected by the stated
    tie-breaks: lowest max-latency candidate, then fewest stages, then the
    lexicographically smallest sequence of (last layer, shape index)), and
    T_of(c) = min over plans with every latency <= c of sum + (B - 1) * c."""
    plans = [(st, lat, sum(lat), max(lat)) for st, lat in enumerate_plans(table, K, D, sizes)]

    def T_of(c):
        best = None
        for st, lat, tot, mx in plans:
            if mx <= c and (best is None or tot < best):
                best = tot
        return None if best is None else best + (B - 1) * c

    if not plans:
        return dict(T_star=None, t_max=None, stages=None, T_of=T_of, plans=plans)
    T_star = min(tot + (B - 1) * mx for _, _, tot, mx in plans)
    return dict(T_star=T_star, T_of=T_of, plans=plans)


def select_plan(plans, c_star):
    """Among plans admissible at c_star with minimal latency sum: fewest stages, then the
    lexicographically smallest ((last layer, shape), ...) sequence in pipeline order."""
    adm = [(st, tot) for st, lat, tot, mx in plans if mx <= c_star]
    m = min(tot for _, tot in adm)
    best = [st for st, tot in adm if tot == m]
    ns = min(len(st) for st in best)
    best = [st for st in best if len(st) == ns]
    best.sort(key=lambda st: [(i, q) for (_, i, q) in st])
    return best[0]
