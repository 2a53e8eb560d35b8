"""ctypes wrapper around the CPU oracle (``alpa_dp_oracle.c``, ``alpa_table_oracle.c``,
``alpa_cluster_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, the smoke check and the
benchmark's ``cpu_baseline`` leg.  It never imports the HIP package and the HIP
package never imports it.  This file marshals arguments; every step of the method
(Eq. 3, Eq. 4, Alg. 1's candidate loop) is in the C file.  The one exception is
``solve_parallel``, a thread-per-candidate driver that re-applies Alg. 1's break and
strict-< selection to per-candidate values computed by the C code; a CPU test holds
it equal to the sequential C loop.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "alpa_dp_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_SRC_TABLE = os.path.join(_HERE, "alpa_table_oracle.c")
_LIB_TABLE = os.path.join(_HERE, "libtable_oracle.so")
_SRC_CLUSTER = os.path.join(_HERE, "alpa_cluster_oracle.c")
_LIB_CLUSTER = os.path.join(_HERE, "libcluster_oracle.so")

INF64 = np.iinfo(np.int64).max
INF32 = np.iinfo(np.int32).max
MAX_K = 256


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, -O2, no threads)."""
    for src, out in ((_SRC, _LIB), (_SRC_TABLE, _LIB_TABLE), (_SRC_CLUSTER, _LIB_CLUSTER)):
        if force or not os.path.exists(out) or os.path.getmtime(out) < os.path.getmtime(src):
            subprocess.check_call(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-Wall",
                                   "-o", out, src])
    return _LIB


class _Plan(ctypes.Structure):
    _fields_ = [("T_star", ctypes.c_int64),
                ("t_max", ctypes.c_int32),
                ("num_stages", ctypes.c_int32),
                ("n_evaluated", ctypes.c_int32),
                ("first_layer", ctypes.c_int32 * (MAX_K + 1)),
                ("shape_idx", ctypes.c_int32 * MAX_K)]


@dataclass
class Plan:
    T_star: int
    t_max: int
    num_stages: int
    n_evaluated: int
    first_layer: list      # len num_stages + 1, 0-based; stage p = [first[p], first[p+1])
    shape_idx: list        # len num_stages

    def key(self):
        return (self.T_star, self.t_max, self.num_stages, tuple(self.first_layer),
                tuple(self.shape_idx))


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        assert L.orc_sizeof_plan() == ctypes.sizeof(_Plan)
        assert L.orc_max_k() == MAX_K
        _lib = L
    return _lib


_lib_table = None


def lib_table():
    global _lib_table
    if _lib_table is None:
        build()
        _lib_table = ctypes.CDLL(_LIB_TABLE)
    return _lib_table


def build_table(t_l, mem_stage, mem_act, mem_device: int) -> np.ndarray:
    """t_intra[s-1][k][i][q] from profiled options [k][i][q][o] (Sec. 5.2, Eq. 5, Alg. 1)."""
    t_l = np.ascontiguousarray(t_l, dtype=np.int32)
    mem_stage = np.ascontiguousarray(mem_stage, dtype=np.int64)
    mem_act = np.ascontiguousarray(mem_act, dtype=np.int64)
    K, K2, S, O = t_l.shape
    assert K == K2 and mem_stage.shape == t_l.shape and mem_act.shape == t_l.shape
    table = np.empty((K, K, K, S), dtype=np.int32)
    rc = lib_table().orc_build_table(_i32p(t_l), _i64p(mem_stage), _i64p(mem_act), K, S, O,
                                     ctypes.c_int64(int(mem_device)), _i32p(table))
    if rc != 0:
        raise RuntimeError(f"orc_build_table failed: {rc}")
    return table


def equal_layer_table(table) -> np.ndarray:
    """The "Equal layer" variant of the ablation study (Sec. 8.3: the DP restricted to the same
    number of layers for all stages), stated on the table: with s stages from first layer k to
    the last, each has (K - k) / s layers, so only such entries stay finite.  Plain loops."""
    table = np.array(table, dtype=np.int32, copy=True)
    K = table.shape[0]
    for s in range(1, K + 1):
        for k in range(K):
            for i in range(K):
                rest = K - k
                if rest % s != 0 or (i - k + 1) * s != rest:
                    table[s - 1, k, i, :] = INF32
    return table


_lib_cluster = None


def cluster_exact(flop, src, dst, nbytes, L: int, delta_ppm: int):
    """Operator clustering (Eq. 6) with the tie-break over whole clusterings: the smallest sum
    of squared per-layer FLOP among all clusterings that reach the optimal G."""
    return cluster(flop, src, dst, nbytes, L, delta_ppm, _fn="orc_cluster_exact")


def cluster(flop, src, dst, nbytes, L: int, delta_ppm: int, _fn: str = "orc_cluster"):
    """Operator clustering (Eq. 6).  Returns (G, V, first_op list of L + 1) or (INF64, 0, [])."""
    global _lib_cluster
    if _lib_cluster is None:
        build()
        _lib_cluster = ctypes.CDLL(_LIB_CLUSTER)
    flop = np.ascontiguousarray(flop, dtype=np.int32)
    src = np.ascontiguousarray(src, dtype=np.int32)
    dst = np.ascontiguousarray(dst, dtype=np.int32)
    nbytes = np.ascontiguousarray(nbytes, dtype=np.int64)
    assert src.size == dst.size == nbytes.size
    G, V = ctypes.c_int64(), ctypes.c_int64()
    first = np.zeros(int(L) + 1, dtype=np.int32)
    rc = getattr(_lib_cluster, _fn)(_i32p(flop), _i32p(src), _i32p(dst), _i64p(nbytes),
                                    int(src.size), int(flop.size), int(L), int(delta_ppm),
                                    ctypes.byref(G), ctypes.byref(V), _i32p(first))
    if rc != 0:
        raise RuntimeError(f"{_fn} failed: {rc}")
    if G.value == INF64:
        return INF64, 0, []
    return int(G.value), int(V.value), [int(x) for x in first]


def _i32p(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _i64p(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))


def _prep(table, shapes):
    table = np.ascontiguousarray(table, dtype=np.int32)
    shapes = np.ascontiguousarray(shapes, dtype=np.int32)
    K = table.shape[0]
    assert table.shape[:3] == (K, K, K) and table.shape[3] == shapes.shape[0]
    return table, shapes, K, shapes.shape[0]


def _plan_out(p: _Plan) -> Plan:
    ns = p.num_stages
    return Plan(int(p.T_star), int(p.t_max), int(ns), int(p.n_evaluated),
                [int(p.first_layer[j]) for j in range(ns + 1)] if ns else [],
                [int(p.shape_idx[j]) for j in range(ns)])


def sort_dedup(v) -> np.ndarray:
    v = np.array(v, dtype=np.int32, copy=True)
    n = lib().orc_sort_dedup(_i32p(v), int(v.size))
    return v[:n].copy()


def all_candidates(table, shapes) -> np.ndarray:
    table, shapes, K, S = _prep(table, shapes)
    out = np.empty(table.size, dtype=np.int32)
    n = lib().orc_all_candidates(_i32p(table), K, S, _i32p(out))
    return out[:n].copy()


def quantiles(v, Q: int) -> np.ndarray:
    v = np.ascontiguousarray(v, dtype=np.int32)
    out = np.empty(max(int(v.size), Q), dtype=np.int32)
    n = lib().orc_quantiles(_i32p(v), int(v.size), int(Q), _i32p(out))
    return out[:n].copy()


def solve(table, N, M, B, shapes, cand, prune: bool):
    """Alg. 1's DP loop, sequential.  cand ascending distinct.  Returns (T[C], Plan)."""
    table, shapes, K, S = _prep(table, shapes)
    cand = np.ascontiguousarray(cand, dtype=np.int32)
    T = np.empty(cand.size, dtype=np.int64)
    p = _Plan()
    rc = lib().orc_solve(_i32p(table), K, int(N), int(M), int(B), _i32p(shapes), S,
                         _i32p(cand), int(cand.size), int(bool(prune)), _i64p(T),
                         ctypes.byref(p))
    if rc != 0:
        raise RuntimeError(f"orc_solve failed: {rc}")
    return T, _plan_out(p)


def eval_candidates(table, N, M, B, shapes, cand, threads: int = 1):
    """T*(c) and s_c for every candidate, no pruning.  ``threads`` > 1 runs the same C
    function on slices of the candidate list (candidates are independent)."""
    table, shapes, K, S = _prep(table, shapes)
    cand = np.ascontiguousarray(cand, dtype=np.int32)
    C = int(cand.size)
    T = np.full(C, INF64, dtype=np.int64)
    sb = np.zeros(C, dtype=np.int32)
    L = lib()

    def run(j0, j1):
        rc = L.orc_eval_candidates(_i32p(table), K, int(N), int(M), int(B), _i32p(shapes), S,
                                   _i32p(cand), j0, j1, _i64p(T), _i32p(sb))
        if rc != 0:
            raise RuntimeError(f"orc_eval_candidates failed: {rc}")

    if threads <= 1 or C < 2:
        run(0, C)
    else:
        # small slices, dealt dynamically: large candidates cost more than small ones
        step = max(1, min(16, C // (threads * 4) or 1))
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(lambda j0: run(j0, min(C, j0 + step)), range(0, C, step)))
    return T, sb


def plan_for(table, N, M, B, shapes, c: int) -> Plan:
    table, shapes, K, S = _prep(table, shapes)
    p = _Plan()
    rc = lib().orc_plan_for(_i32p(table), K, int(N), int(M), int(B), _i32p(shapes), S,
                            int(c), ctypes.byref(p))
    if rc != 0:
        raise RuntimeError(f"orc_plan_for failed: {rc}")
    return _plan_out(p)


def fill_F(table, N, M, shapes, c: int):
    """F[s][k][d] of Eq. 3 for one candidate: arrays of shape (Smax+1, K+2, D+1),
    layers 1-based on axis 1.  Returns (F, Ai, Aq)."""
    table, shapes, K, S = _prep(table, shapes)
    D = int(N) * int(M)
    Smax = min(K, D)
    a = np.ascontiguousarray(shapes[:, 0] * shapes[:, 1], dtype=np.int32)
    F = np.empty((Smax + 1, K + 2, D + 1), dtype=np.int64)
    Ai = np.empty(F.shape, dtype=np.int32)
    Aq = np.empty(F.shape, dtype=np.int32)
    lib().orc_fill_F(_i32p(table), K, D, S, _i32p(a), ctypes.c_int32(int(c)), Smax,
                     _i64p(F), _i32p(Ai), _i32p(Aq))
    return F, Ai, Aq


def solve_parallel(table, N, M, B, shapes, cand, prune: bool, threads: int):
    """Same result as ``solve`` by definition of the sequential rule, with the per-candidate
    bodies run on several threads: evaluate every T*(c), then apply Alg. 1's break and
    strict-< selection in candidate order, then recover the plan of the winner."""
    T, _ = eval_candidates(table, N, M, B, shapes, cand, threads)
    best, bj, processed = INF64, -1, 0
    for j in range(len(cand)):
        if prune and best != INF64 and int(B) * int(cand[j]) >= best:
            break
        processed += 1
        if T[j] < best:
            best, bj = int(T[j]), j
    T[processed:] = INF64
    if bj < 0:
        return T, Plan(INF64, 0, 0, processed, [], [])
    p = plan_for(table, N, M, B, shapes, int(cand[bj]))
    p.n_evaluated = processed
    return T, p
