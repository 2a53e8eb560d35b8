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
    terms: dict = field(default=None)              # formula workloads: the table's ingredients

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


def _a2a_us(a: int) -> int:
    """All-to-all time of one expert layer on a devices: the tabulated values (300 log2 a,
    rounded) for the sizes of the 8 x 8 mesh, the same formula beyond."""
    if a <= 1:
        return 0
    if a in _A2A_US:
        return _A2A_US[a]
    import math
    return int(math.floor(300.0 * math.log2(a) + 0.5))


def _formula_table(K, shapes, cost, mem, act_per_layer, cap, *, expert=None,
                   act_mode="const", terms=None):
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
        a2a = np.asarray([_a2a_us(int(x)) for x in a], dtype=np.int64)
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
    if terms is not None:
        terms.update(lat=lat, msum=msum, actv=actv, cap=int(cap), a=a, valid=valid)
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
        terms = {}
        table = _formula_table(K, shapes, cost, mem, 1, 16, terms=terms)
        return Workload("tiny", K, N, M, B, shapes, table, "all", 0, False, seed,
                        cost, mem, np.full(K, 1, np.int64), terms)
    if idx == 2:
        K, N, M, B, seed = 24, 2, 8, 32, 1
        rng = SplitMix64(seed)
        cost = np.zeros(K, np.int64); mem = np.zeros(K, np.int64)
        for l in range(K):
            cost[l] = rng.uint(900, 1100); mem[l] = rng.uint(3, 5)
        shapes = submesh_shapes(N, M)
        terms = {}
        table = _formula_table(K, shapes, cost, mem, 2, 80, terms=terms)
        return Workload("gpt", K, N, M, B, shapes, table, "all", 0, True, seed,
                        cost, mem, np.full(K, 2, np.int64), terms)
    if idx == 3:
        K, N, M, B, seed = 48, 8, 8, 64, 2
        rng = SplitMix64(seed)
        cost = np.zeros(K, np.int64); mem = np.zeros(K, np.int64)
        for l in range(K):
            cost[l] = rng.uint(1800, 2200); mem[l] = rng.uint(6, 10)
        shapes = submesh_shapes(N, M)
        terms = {}
        table = _formula_table(K, shapes, cost, mem, 4, 80, terms=terms)
        return Workload("large", K, N, M, B, shapes, table, "quantiles", 4096, False, seed,
                        cost, mem, np.full(K, 4, np.int64), terms)
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
        terms = {}
        table = _formula_table(K, shapes, cost, mem, 3, 80, expert=expert, terms=terms)
        return Workload("moe", K, N, M, B, shapes, table, "quantiles", 4096, False, seed,
                        cost, mem, np.full(K, 3, np.int64), terms)
    if idx == 5:
        K, N, M, B, seed = 64, 8, 8, 32, 4
        rng = SplitMix64(seed)
        cost = np.zeros(K, np.int64); mem = np.zeros(K, np.int64); act = np.zeros(K, np.int64)
        for l in range(K):
            cost[l] = _round_half_away(3000.0 * 0.97 ** l) + rng.uint(0, 200)
            mem[l] = _round_half_away(1.0 + 0.5 * 1.06 ** l)
            act[l] = _round_half_away(12.0 * 0.95 ** l)
        shapes = submesh_shapes(N, M)
        terms = {}
        table = _formula_table(K, shapes, cost, mem, act, 80, act_mode="max", terms=terms)
        return Workload("wrn", K, N, M, B, shapes, table, "all", 0, False, seed,
                        cost, mem, act, terms)
    raise ValueError("workload index must be 1..5")


def deep_model_problem(seed: int, K: int, N: int, M: int, B: int = 64) -> Workload:
    """A formula table of the MoE-like kind for any layer count (deeper models than the five
    numbered workloads: up to 128 layers), with the memory cap scaled to the depth."""
    rng = SplitMix64(seed)
    cost = np.zeros(K, np.int64); mem = np.zeros(K, np.int64)
    expert = np.zeros(K, np.int64)
    for l in range(K):
        if l % 2 == 0:
            cost[l] = rng.uint(500, 700); mem[l] = rng.uint(2, 3)
        else:
            cost[l] = rng.uint(2000, 2800); mem[l] = rng.uint(16, 24)
            expert[l] = 1
    shapes = submesh_shapes(N, M)
    terms = {}
    cap = max(24, (80 * K * 64) // (64 * N * M))
    table = _formula_table(K, shapes, cost, mem, 3, cap, expert=expert, terms=terms)
    return Workload("deep", K, N, M, B, shapes, table, "quantiles", 4096, False, seed,
                    cost, mem, np.full(K, 3, np.int64), terms)


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


def many_stage_problem(seed: int, K: int, N: int, M: int, B: int = 512) -> Workload:
    """A table on which more devices buy no speed (latency = 1000 per layer + 40 per extra
    device + noise below 50) and many microbatches: the optimum cuts the model into nearly as
    many one-device stages as layers or devices allow, so stage counts far above those of
    the model-like workloads are exercised."""
    rng = np.random.default_rng(seed)
    shapes = submesh_shapes(N, M)
    S = shapes.shape[0]
    a = shapes[:, 0].astype(np.int64) * shapes[:, 1]
    kk = np.arange(K)[:, None]
    ii = np.arange(K)[None, :]
    lat = 1000 * (ii - kk + 1)[:, :, None] + 40 * (a - 1)[None, None, :]
    lat = lat + rng.integers(0, 50, size=(K, K, S))
    table = np.broadcast_to(lat[None], (K, K, K, S)).copy()
    table[:, ii < kk, :] = int(INF_I32)
    return Workload(f"stages{seed}", K, N, M, B, shapes.astype(np.int32),
                    np.ascontiguousarray(table.astype(np.int32)), "quantiles", 16, False, seed)


# ---------------------------------------------------------------------------------------------
# Profiled options: the inputs of the table-construction step (Sec. 5.2, Eq. 5; Alg. 1's
# "run the intra-op pass" loop nest).  Only inputs are made here; the step itself (pick the
# fastest option that fits, per s) is in the oracle and in the HIP library.

@dataclass
class Profiles:
    K: int
    S: int
    O: int
    t_l: np.ndarray             # int32 [K, K, S, O] microseconds, INF = option absent
    mem_stage: np.ndarray       # int64 [K, K, S, O] bytes per device
    mem_act: np.ndarray         # int64 [K, K, S, O] bytes per device and in-flight microbatch
    mem_device: int             # bytes


def single_option_profiles(w: Workload) -> Profiles:
    """One option per (stage, submesh) whose figures restate a formula workload: the workload's
    rule "sum mem + s * act <= cap * a" becomes "mem_stage + s * mem_act <= mem_device" with
    mem_stage = sum mem + (BIG - cap * a), mem_act = act, mem_device = BIG."""
    t = w.terms
    K, S = w.K, w.S
    big = int(t["cap"]) * int(t["a"].max())
    valid = t["valid"][:, :, None, None]
    t_l = np.where(valid, t["lat"][:, :, :, None], int(INF_I32)).astype(np.int32)
    mem_stage = (t["msum"][:, :, None] + (big - t["cap"] * t["a"])[None, None, :])[..., None]
    mem_act = np.broadcast_to(t["actv"][:, :, None, None], (K, K, S, 1))
    return Profiles(K, S, 1, np.ascontiguousarray(t_l),
                    np.ascontiguousarray(mem_stage.astype(np.int64)),
                    np.ascontiguousarray(mem_act.astype(np.int64)), big)


def make_profiles(idx: int, n_options: int = 6) -> Profiles:
    """Several options per (stage, submesh) for formula workload ``idx``: option o is slower and
    leaner than option o - 1 (more sharding / rematerialisation): latency x (100 + 9 o + U[0,5]) %,
    memory x (16 - 2 o) / 16 with a floor of 1/4, in bytes per device (1 MiB units, ceil-divided by
    the device count); about 8 % of the options are absent.  mem_device = cap MiB."""
    w = make_workload(idx)
    t = w.terms
    K, S, O = w.K, w.S, int(n_options)
    rng = np.random.default_rng(1000 + w.seed)
    a = t["a"].astype(np.int64)
    lat = t["lat"].astype(np.int64)[:, :, :, None]                              # [K,K,S,1]
    o = np.arange(O, dtype=np.int64)[None, None, None, :]
    jitter = rng.integers(0, 6, size=(K, K, S, O), dtype=np.int64)
    t_l = lat * (100 + 9 * o + jitter) // 100
    absent = rng.random(size=(K, K, S, O)) < 0.08
    valid = t["valid"][:, :, None, None]
    t_l = np.where(valid & ~absent, t_l, int(INF_I32)).astype(np.int32)
    lean = np.maximum(16 - 2 * o, 4)                                            # sixteenths
    mib = 1 << 20
    ms = t["msum"].astype(np.int64)[:, :, None, None] * mib * lean              # x16, all devices
    ma = t["actv"].astype(np.int64)[:, :, None, None] * mib * lean
    div = 16 * a[None, None, :, None]
    mem_stage = (ms + div - 1) // div
    mem_act = np.broadcast_to((ma + div - 1) // div, (K, K, S, O))
    return Profiles(K, S, O, np.ascontiguousarray(t_l), np.ascontiguousarray(mem_stage),
                    np.ascontiguousarray(mem_act), int(t["cap"]) * mib)


def random_profiles(seed: int, K: int, S: int, O: int, *, absent_frac: float = 0.2) -> Profiles:
    """Unstructured profiles: every figure drawn independently, many ties, zero activation
    sizes, options absent with probability ``absent_frac``, and a device size in the middle of
    the range of requirements so that the fitting set changes with s."""
    rng = np.random.default_rng(seed)
    t_l = rng.integers(1, 60, size=(K, K, S, O), dtype=np.int64)
    t_l[rng.random(size=t_l.shape) < absent_frac] = int(INF_I32)
    kk = np.arange(K)[:, None]
    ii = np.arange(K)[None, :]
    t_l[ii < kk] = int(INF_I32)
    mem_stage = rng.integers(0, 40, size=t_l.shape, dtype=np.int64)
    mem_act = rng.integers(0, 6, size=t_l.shape, dtype=np.int64)
    mem_device = int(rng.integers(20, 40 + 3 * K))
    return Profiles(K, S, O, np.ascontiguousarray(t_l.astype(np.int32)), mem_stage, mem_act,
                    mem_device)


# ---------------------------------------------------------------------------------------------
# Operator graphs: the inputs of the operator-clustering step (Sec. 5.2, Eq. 6).  Inputs only.

@dataclass
class OpGraph:
    K: int
    flop: np.ndarray            # int32 [K], caller's unit (here MFLOP), total < 2^31
    src: np.ndarray             # int32 [E] producer (0-based), src < dst
    dst: np.ndarray             # int32 [E] consumer
    nbytes: np.ndarray          # int64 [E]


def make_op_graph(seed: int, n_blocks: int) -> OpGraph:
    """Flattened transformer-like graph: an embedding, ``n_blocks`` blocks of 12 operators
    (norm, qkv, scores, softmax, context, proj, add, norm, mlp-up, gelu, mlp-down, add) and a
    head.  Matrix products carry the FLOP (with +-10 % jitter), element-wise operators almost
    none; every operator feeds the next one with an activation-sized tensor (the score tensors
    are 4x larger), and each residual ``add`` also reads the block's input (a skip edge)."""
    rng = np.random.default_rng(seed)
    act = 8 << 20                                     # bytes of one activation tensor
    heavy = {1: 3000, 2: 500, 4: 500, 5: 1000, 8: 4000, 10: 4000}
    flop, src, dst, nb = [40], [], [], []            # embedding
    for b in range(n_blocks):
        base = len(flop)
        for j in range(12):
            f = heavy.get(j, 2)
            flop.append(int(f * (0.9 + 0.2 * rng.random())) if f > 2 else int(rng.integers(1, 4)))
            src.append(base + j - 1)
            dst.append(base + j)
            nb.append(act * (4 if j in (3, 4) else 1) + int(rng.integers(0, 4096)))
        # residual connections: block input -> first add, first add -> second add
        src += [base - 1, base + 6]
        dst += [base + 6, base + 11]
        nb += [act, act]
        # qkv output is also read by the context product
        src.append(base + 1); dst.append(base + 4); nb.append(act)
    flop.append(2500)                                 # head
    src.append(len(flop) - 2); dst.append(len(flop) - 1); nb.append(act)
    return OpGraph(len(flop), np.asarray(flop, np.int32), np.asarray(src, np.int32),
                   np.asarray(dst, np.int32), np.asarray(nb, np.int64))


def random_op_graph(seed: int, K: int, E: int, *, flop_hi: int = 9, bytes_hi: int = 6) -> OpGraph:
    """Unstructured graph: independent FLOP figures (zeros allowed), E random forward edges
    (parallel edges allowed) with small byte counts, so ties are frequent."""
    rng = np.random.default_rng(seed)
    flop = rng.integers(0, flop_hi + 1, size=K).astype(np.int32)
    if K >= 2 and E > 0:
        u = rng.integers(0, K - 1, size=E)
        v = u + 1 + (rng.integers(0, K, size=E) % (K - 1 - u))
        nb = rng.integers(0, bytes_hi + 1, size=E)
    else:
        u = v = nb = np.zeros(0, np.int64)
    return OpGraph(K, flop, u.astype(np.int32), v.astype(np.int32), nb.astype(np.int64))
