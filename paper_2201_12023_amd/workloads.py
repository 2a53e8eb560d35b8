"""Seeded synthetic inputs for the stage-slicing dynamic program (Sec. 5.2).

This module only *makes inputs*: per-stage latency tables ``t_intra`` (Sec. 5.2,
the quantity the intra-op pass reports for every stage / submesh / s triple),
the submesh-shape list (Alg. 1, the ``submesh_shapes`` set) and the scalar
problem parameters.  It holds none of the method's arithmetic (no recurrence,
no candidate selection, no pruning) so that the CPU oracle and the HIP library
can both be fed from it without sharing any code of the method itself.

The paper's real tables were profiled on its own cluster and never published;
the five seeded formula workloads below stand in for them.  Their sizes follow
the paper's model and cluster sizes (Appendix B layer counts, 1..64 devices).

Table layout (the layout of the C ABI): C-order ``[s-1][k][i][q]`` with extents
``K x K x K x S``; ``k``/``i`` are the 0-based first/last layer of a stage,
``q`` indexes ``shapes``; entries with ``i < k`` are unused and set to ``INF``;
``INF = INT32_MAX`` marks a memory-infeasible entry (Eq. 5).  Values are int32
microseconds.

Random numbers: splitmix64 seeded with the workload seed; ``U_int[a, b]`` is
``a + next() % (b - a + 1)``; draw order per layer ``l``: cost, then memory
(workload 5 draws only its cost jitter).
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

INF_I32 = np.int32(2**31 - 1)

_MASK64 = (1 << 64) - 1


class SplitMix64:
    """Public-domain splitmix64 counter-based generator (Steele et al.)."""

    def __init__(self, seed: int):
        self.state = seed & _MASK64

    def next(self) -> int:
        self.state = (self.state + 0x9E3779B97F4A7C15) & _MASK64
        z = self.state
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK64
        return z ^ (z >> 31)

    def uint(self, a: int, b: int) -> int:
        return a + self.next() % (b - a + 1)


@dataclass
class Workload:
    name: str
    K: int
    N: int
    M: int
    B: int
    shapes: np.ndarray          # int32 [S, 2] rows (n, m)
    table: np.ndarray           # int32 [K, K, K, S]  = [s-1][k][i][q]
    candidates: str             # "all" or "quantiles"
    n_quantiles: int            # used when candidates == "quantiles"
    prune: bool
    seed: int
    layer_cost: np.ndarray = field(default=None)   # int64 [K], for the run log
    layer_mem: np.ndarray = field(default=None)    # int64 [K]
    layer_act: np.ndarray = field(default=None)    # int64 [K]

    @property
    def S(self) -> int:
        return int(self.shapes.shape[0])

    @property
    def D(self) -> int:
        return self.N * self.M

    @property
    def sizes(self) -> np.ndarray:
        return (self.shapes[:, 0].astype(np.int64) * self.shapes[:, 1]).astype(np.int32)


def submesh_shapes(N: int, M: int) -> np.ndarray:
    """The shape family of Sec. 5.2 / Alg. 1: (1, 2^p) for 2^p <= M, then (n, M), n = 2..N."""
    out = []
    p = 1
    while p <= M:
        out.append((1, p))
        p *= 2
    for n in range(2, N + 1):
        out.append((n, M))
    return np.asarray(out, dtype=np.int32)


# round(300 * log2(a)) for the device counts the 8x8 family can produce
_A2A_US = {1: 0, 2: 300, 4: 600, 8: 900, 16: 1200, 24: 1375, 32: 1500,
           40: 1597, 48: 1675, 56: 1742, 64: 1800}


def _formula_table(K, shapes, cost, mem, act_per_layer, cap, *, expert=None,
                   act_mode="const"):
    """t(k..i, q, s) = ceil(sum c / a) + 50 (a - 1) + (n > 1 ? 400 : 0) [+ experts * a2a(a)],
    INF iff sum mem + s * act > cap * a  (integer-exact, no division)."""
    S = shapes.shape[0]
    a = shapes[:, 0].astype(np.int64) * shapes[:, 1].astype(np.int64)          # [S]
    inter = np.where(shapes[:, 0] > 1, 400, 0).astype(np.int64)                # [S]
    pc = np.concatenate([[0], np.cumsum(cost.astype(np.int64))])
    pm = np.concatenate([[0], np.cumsum(mem.astype(np.int64))])
    kk = np.arange(K)[:, None]
    ii = np.arange(K)[None, :]
    valid = ii >= kk                                                           # [K, K]
    csum = np.where(valid, pc[ii + 1] - pc[kk], 0)                             # [K, K]
    msum = np.where(valid, pm[ii + 1] - pm[kk], 0)
    lat = (csum[:, :, None] + a[None, None, :] - 1) // a[None, None, :]
    lat = lat + 50 * (a - 1)[None, None, :] + inter[None, None, :]
    if expert is not None:
        pe = np.concatenate([[0], np.cumsum(expert.astype(np.int64))])
        ecnt = np.where(valid, pe[ii + 1] - pe[kk], 0)
        a2a = np.asarray([_A2A_US[int(x)] if x > 1 else 0 for x in a], dtype=np.int64)
        lat = lat + ecnt[:, :, None] * a2a[None, None, :]
    if act_mode == "const":
        actv = np.full((K, K), int(act_per_layer), dtype=np.int64)
    else:  # max of the per-layer activation sizes inside the stage
        actv = np.zeros((K, K), dtype=np.int64)
        for k in range(K):
            run = 0
            for i in range(k, K):
                run = max(run, int(act_per_layer[i]))
                actv[k, i] = run
    s = np.arange(1, K + 1, dtype=np.int64)[:, None, None, None]               # [K,1,1,1]
    need = msum[None, :, :, None] + s * actv[None, :, :, None]                 # [K,K,K,1]
    feas = need <= (cap * a)[None, None, None, :]
    table = np.where(feas & valid[None, :, :, None], lat[None, :, :, :], int(INF_I32))
    assert table[table != int(INF_I32)].max() < 2**30
    return np.ascontiguousarray(table.astype(np.int32))


def make_workload(idx: int) -> Workload:
    """Workloads 1..5 (1-based), sizes and distributions as listed in the module docstring
    of the benchmark description: Tiny, GPT-like, Large uniform, MoE-like, Wide-ResNet-like."""
    if idx == 1:
        K, N, M, B, seed = 8, 1, 4, 8, 0
        rng = SplitMix64(seed)
        cost = np.zeros(K, np.int64); mem = np.zeros(K, np.int64)
        for l in range(K):
            cost[l] = rng.uint(200, 2000); mem[l] = rng.uint(1, 8)
        shapes = submesh_shapes(N, M)
        table = _formula_table(K, shapes, cost, mem, 1, 16)
        return Workload("tiny", K, N, M, B, shapes, table, "all", 0, False, seed,
                        cost, mem, np.full(K, 1, np.int64))
    if idx == 2:
        K, N, M, B, seed = 24, 2, 8, 32, 1
        rng = SplitMix64(seed)
        cost = np.zeros(K, np.int64); mem = np.zeros(K, np.int64)
        for l in range(K):
            cost[l] = rng.uint(900, 1100); mem[l] = rng.uint(3, 5)
        shapes = submesh_shapes(N, M)
        table = _formula_table(K, shapes, cost, mem, 2, 80)
        return Workload("gpt", K, N, M, B, shapes, table, "all", 0, True, seed,
                        cost, mem, np.full(K, 2, np.int64))
    if idx == 3:
        K, N, M, B, seed = 48, 8, 8, 64, 2
        rng = SplitMix64(seed)
        cost = np.zeros(K, np.int64); mem = np.zeros(K, np.int64)
        for l in range(K):
            cost[l] = rng.uint(1800, 2200); mem[l] = rng.uint(6, 10)
        shapes = submesh_shapes(N, M)
        table = _formula_table(K, shapes, cost, mem, 4, 80)
        return Workload("large", K, N, M, B, shapes, table, "quantiles", 4096, False, seed,
                        cost, mem, np.full(K, 4, np.int64))
    if idx == 4:
        K, N, M, B, seed = 64, 8, 8, 128, 3
        rng = SplitMix64(seed)
        cost = np.zeros(K, np.int64); mem = np.zeros(K, np.int64)
        expert = np.zeros(K, np.int64)
        for l in range(K):
            if l % 2 == 0:   # dense
                cost[l] = rng.uint(500, 700); mem[l] = rng.uint(2, 3)
            else:            # expert
                cost[l] = rng.uint(2000, 2800); mem[l] = rng.uint(16, 24)
                expert[l] = 1
        shapes = submesh_shapes(N, M)
        table = _formula_table(K, shapes, cost, mem, 3, 80, expert=expert)
        return Workload("moe", K, N, M, B, shapes, table, "quantiles", 4096, False, seed,
                        cost, mem, np.full(K, 3, np.int64))
    if idx == 5:
        K, N, M, B, seed = 64, 8, 8, 32, 4
        rng = SplitMix64(seed)
        cost = np.zeros(K, np.int64); mem = np.zeros(K, np.int64); act = np.zeros(K, np.int64)
        for l in range(K):
            cost[l] = _round_half_away(3000.0 * 0.97 ** l) + rng.uint(0, 200)
            mem[l] = _round_half_away(1.0 + 0.5 * 1.06 ** l)
            act[l] = _round_half_away(12.0 * 0.95 ** l)
        shapes = submesh_shapes(N, M)
        table = _formula_table(K, shapes, cost, mem, act, 80, act_mode="max")
        return Workload("wrn", K, N, M, B, shapes, table, "all", 0, False, seed,
                        cost, mem, act)
    raise ValueError("workload index must be 1..5")


def _round_half_away(x: float) -> int:
    import math
    return int(math.floor(abs(x) + 0.5)) * (1 if x >= 0 else -1)


def random_problem(seed: int, K: int, N: int, M: int, *, S_extra_dup: bool = False,
                   inf_frac: float = 0.2, value_hi: int = 40, B: int | None = None):
    """Small unstructured problem for brute-force / parity tests: every table entry drawn
    independently (so it is *not* monotone in the stage length), a fraction ``inf_frac`` set
    to INF, and a narrow value range so that equal values (ties) are frequent."""
    rng = np.random.default_rng(seed)
    shapes = submesh_shapes(N, M)
    if S_extra_dup:
        shapes = np.concatenate([shapes, shapes[:1]], axis=0)
    S = shapes.shape[0]
    table = rng.integers(1, value_hi + 1, size=(K, K, K, S), dtype=np.int64)
    table[rng.random(size=table.shape) < inf_frac] = int(INF_I32)
    kk = np.arange(K)[:, None]
    ii = np.arange(K)[None, :]
    table[:, ii < kk, :] = int(INF_I32)
    if B is None:
        B = int(rng.integers(1, 9))
    return Workload(f"rand{seed}", K, N, M, B, shapes.astype(np.int32),
                    np.ascontiguousarray(table.astype(np.int32)), "all", 0, False, seed)
