"""Thin ctypes binding over the C ABI in ``include/alpa_dp.h`` (argument marshalling only).

Same names as the C entry points.  PyTorch is used for device memory (``torch.Tensor``
arguments of ``alpa_dp_solve_dev``) and streams; every step of the method runs in the HIP
kernels of ``libalpa_dp.so``.  There is no CPU fallback: loading fails loudly if the
library has not been built.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libalpa_dp.so")

MAX_K = 256
MAX_SWEEP = 256
MAX_OPTIONS = 32
CLUSTER_MAX_OPS = 4096
CLUSTER_STATIC_MAX_OPS = 512
INF_I32 = 2**31 - 1
INF_I64 = 2**63 - 1
ALPA_DP_PRUNE = 1
ALPA_DP_GENERIC = 2
ALPA_DP_COUNT_WORK = 4
ALPA_DP_TUNE_CANDIDATES_PER_WG = 1
ALPA_DP_TUNE_DISTINCT_BY_SORT = 2
ALPA_DP_TUNE_WG_PER_CU = 3
ALPA_DP_TUNE_WORKGROUPS = 4
ALPA_DP_TUNE_LANE_GROUPS = 5

SYMBOLS = ["alpa_dp_create", "alpa_dp_create_from_profiles", "alpa_dp_get_table",
           "alpa_dp_restrict_equal_layers", "alpa_dp_set_stream", "alpa_dp_set_B", "alpa_dp_set_tuning", "alpa_dp_count_candidates",
           "alpa_dp_solve", "alpa_dp_solve_dev", "alpa_dp_solve_sweep", "alpa_dp_candidates",
           "alpa_dp_best",
           "alpa_dp_last_timing", "alpa_dp_last_counters", "alpa_dp_destroy",
           "alpa_dp_last_error", "alpa_cluster_layers", "alpa_cluster_layers_exact", "alpa_cluster_layers_static", "alpa_place_submeshes", "alpa_dp_measure_valu_peak"]


class alpa_shape_t(ctypes.Structure):
    _fields_ = [("n", ctypes.c_int32), ("m", ctypes.c_int32)]


class alpa_plan_t(ctypes.Structure):
    _fields_ = [("T_star", ctypes.c_int64),
                ("t_max", ctypes.c_int32),
                ("num_stages", ctypes.c_int32),
                ("n_evaluated", ctypes.c_int32),
                ("first_layer", ctypes.c_int32 * (MAX_K + 1)),
                ("shape_idx", ctypes.c_int32 * MAX_K)]

    def as_dict(self):
        ns = max(0, int(self.num_stages))
        return dict(T_star=int(self.T_star), t_max=int(self.t_max), num_stages=int(self.num_stages),
                    n_evaluated=int(self.n_evaluated),
                    first_layer=[int(self.first_layer[j]) for j in range(ns + 1)] if ns else [],
                    shape_idx=[int(self.shape_idx[j]) for j in range(ns)])


class AlpaDpError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"alpa_dp error {code}: {msg}")
        self.code = code


_lib = None


def load():
    """Load libalpa_dp.so (raises if it is not built; build with
    ``python -m paper_2201_12023_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build the HIP library first "
            "(python -m paper_2201_12023_amd.build); there is no CPU fallback")
    L = ctypes.CDLL(LIB_PATH)
    vp, i32p, i64p = ctypes.c_void_p, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int64)
    L.alpa_dp_create.argtypes = [ctypes.POINTER(vp), vp, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                 ctypes.c_int, ctypes.POINTER(alpa_shape_t), ctypes.c_int]
    L.alpa_dp_create_from_profiles.argtypes = [ctypes.POINTER(vp), vp, vp, vp, ctypes.c_int,
                                               ctypes.c_int64, ctypes.c_int, ctypes.c_int,
                                               ctypes.c_int, ctypes.c_int,
                                               ctypes.POINTER(alpa_shape_t), ctypes.c_int]
    L.alpa_dp_get_table.argtypes = [vp, vp]
    L.alpa_dp_restrict_equal_layers.argtypes = [vp]
    L.alpa_dp_set_stream.argtypes = [vp, vp]
    L.alpa_dp_set_B.argtypes = [vp, ctypes.c_int]
    L.alpa_dp_set_tuning.argtypes = [vp, ctypes.c_int, ctypes.c_int]
    L.alpa_dp_count_candidates.argtypes = [vp, ctypes.POINTER(ctypes.c_int)]
    L.alpa_dp_solve.argtypes = [vp, vp, ctypes.c_int, ctypes.c_uint, vp, vp]
    L.alpa_dp_solve_dev.argtypes = [vp, vp, ctypes.c_int, ctypes.c_uint, vp, vp]
    L.alpa_dp_solve_sweep.argtypes = [vp, vp, ctypes.c_int, ctypes.c_uint, vp, ctypes.c_int, vp]
    L.alpa_dp_candidates.argtypes = [vp, vp, ctypes.c_int, ctypes.POINTER(ctypes.c_int)]
    L.alpa_dp_best.argtypes = [vp, ctypes.POINTER(alpa_plan_t)]
    L.alpa_dp_last_timing.argtypes = [vp] + [ctypes.POINTER(ctypes.c_float)] * 3
    L.alpa_dp_last_counters.argtypes = [vp, ctypes.POINTER(ctypes.c_int), i64p]
    L.alpa_cluster_layers.argtypes = [vp, ctypes.c_int, vp, vp, vp, ctypes.c_int, ctypes.c_int,
                                      ctypes.c_int, i64p, i64p, vp,
                                      ctypes.POINTER(ctypes.c_float)]
    L.alpa_cluster_layers_exact.argtypes = L.alpa_cluster_layers.argtypes
    L.alpa_cluster_layers_static.argtypes = [vp, ctypes.c_int, vp, vp, vp, ctypes.c_int,
                                             ctypes.c_int, ctypes.c_int, vp, vp, vp]
    L.alpa_place_submeshes.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.POINTER(alpa_shape_t),
                                       ctypes.c_int, vp, vp]
    L.alpa_dp_measure_valu_peak.argtypes = [ctypes.POINTER(ctypes.c_double)]
    L.alpa_dp_destroy.argtypes = [vp]
    L.alpa_dp_destroy.restype = None
    L.alpa_dp_last_error.restype = ctypes.c_char_p
    _lib = L
    return L


def _check(rc):
    if rc != 0:
        raise AlpaDpError(rc, load().alpa_dp_last_error().decode())


def alpa_dp_create(cost_table, K, N, M, B, shapes):
    """cost_table: int32 numpy array [K, K, K, S] (host); shapes: int32 [S, 2] rows (n, m)."""
    L = load()
    table = np.ascontiguousarray(cost_table, dtype=np.int32)
    shp = np.ascontiguousarray(shapes, dtype=np.int32).reshape(-1, 2)
    S = shp.shape[0]
    if table.size != K * K * K * S:
        raise ValueError("cost_table must have K*K*K*num_shapes entries")
    arr = (alpa_shape_t * S)(*[alpa_shape_t(int(n), int(m)) for n, m in shp])
    h = ctypes.c_void_p()
    _check(L.alpa_dp_create(ctypes.byref(h), table.ctypes.data, K, N, M, B, arr, S))
    return h


def alpa_dp_create_from_profiles(t_l, mem_stage, mem_act, mem_device, K, N, M, B, shapes):
    """t_l int32 / mem_stage, mem_act int64 numpy arrays [K, K, S, O] (host); the table is built
    on the device."""
    L = load()
    shp = np.ascontiguousarray(shapes, dtype=np.int32).reshape(-1, 2)
    S = shp.shape[0]
    t = np.ascontiguousarray(t_l, dtype=np.int32)
    ms = np.ascontiguousarray(mem_stage, dtype=np.int64)
    ma = np.ascontiguousarray(mem_act, dtype=np.int64)
    if t.size % (K * K * S) != 0 or ms.size != t.size or ma.size != t.size:
        raise ValueError("profile arrays must have K*K*num_shapes*num_options entries each")
    O = t.size // (K * K * S)
    arr = (alpa_shape_t * S)(*[alpa_shape_t(int(n), int(m)) for n, m in shp])
    h = ctypes.c_void_p()
    _check(L.alpa_dp_create_from_profiles(ctypes.byref(h), t.ctypes.data, ms.ctypes.data,
                                          ma.ctypes.data, O, int(mem_device), K, N, M, B, arr, S))
    return h


def alpa_dp_get_table(h, K, S) -> np.ndarray:
    out = np.empty((K, K, K, S), dtype=np.int32)
    _check(load().alpa_dp_get_table(h, out.ctypes.data))
    return out


def alpa_dp_restrict_equal_layers(h):
    _check(load().alpa_dp_restrict_equal_layers(h))


def alpa_dp_set_stream(h, stream):
    """stream: a torch.cuda.Stream (its HIP stream handle is passed down) or a raw handle."""
    raw = getattr(stream, "cuda_stream", stream)
    _check(load().alpa_dp_set_stream(h, ctypes.c_void_p(int(raw))))


def alpa_dp_set_B(h, B):
    _check(load().alpa_dp_set_B(h, int(B)))


def alpa_dp_set_tuning(h, key, value):
    _check(load().alpa_dp_set_tuning(h, int(key), int(value)))


def alpa_dp_count_candidates(h) -> int:
    n = ctypes.c_int()
    _check(load().alpa_dp_count_candidates(h, ctypes.byref(n)))
    return n.value


def alpa_dp_solve(h, tmax, n_tmax=None, flags=0, want_T=True, want_plan=True):
    """tmax: int32 array-like (host) or None.  Returns (T int64 numpy or None, plan dict or None)."""
    L = load()
    if tmax is not None:
        t = np.ascontiguousarray(tmax, dtype=np.int32)
        n = int(t.size) if n_tmax is None else int(n_tmax)
        n_out = n
        tp = t.ctypes.data
    else:
        n = 0 if n_tmax is None else int(n_tmax)
        nd = alpa_dp_count_candidates(h)
        n_out = nd if n == 0 else min(nd, n)
        tp = None
    T = np.full(max(n_out, 1), INF_I64, dtype=np.int64) if want_T else None
    plan = alpa_plan_t() if want_plan else None
    _check(L.alpa_dp_solve(h, tp, n, flags, T.ctypes.data if want_T else None,
                           ctypes.addressof(plan) if want_plan else None))
    return (T[:n_out] if want_T else None), (plan.as_dict() if want_plan else None)


def alpa_dp_solve_dev(h, d_tmax, n_tmax, flags, d_out_T, d_out_plan):
    """Device-pointer variant: arguments are torch CUDA tensors (int32 / int64 / uint8 for the
    plan buffer of ctypes.sizeof(alpa_plan_t) bytes) or None.  Asynchronous."""
    def ptr(t):
        return None if t is None else ctypes.c_void_p(int(t.data_ptr()))
    _check(load().alpa_dp_solve_dev(h, ptr(d_tmax), int(n_tmax), int(flags), ptr(d_out_T),
                                    ptr(d_out_plan)))


def alpa_dp_solve_sweep(h, tmax, B_values, n_tmax=None, flags=0):
    """One plan dict per value of B_values (int32 array-like, host); tmax as for alpa_dp_solve."""
    L = load()
    if tmax is not None:
        t = np.ascontiguousarray(tmax, dtype=np.int32)
        n = int(t.size) if n_tmax is None else int(n_tmax)
        tp = t.ctypes.data
    else:
        n = 0 if n_tmax is None else int(n_tmax)
        tp = None
    B = np.ascontiguousarray(B_values, dtype=np.int32)
    plans = (alpa_plan_t * max(int(B.size), 1))()
    _check(L.alpa_dp_solve_sweep(h, tp, n, flags, B.ctypes.data if B.size else None, int(B.size),
                                 ctypes.addressof(plans)))
    return [plans[b].as_dict() for b in range(int(B.size))]


def alpa_dp_candidates(h) -> np.ndarray:
    L = load()
    n = ctypes.c_int()
    _check(L.alpa_dp_candidates(h, None, 0, ctypes.byref(n)))
    out = np.empty(max(n.value, 1), dtype=np.int32)
    _check(L.alpa_dp_candidates(h, out.ctypes.data, n.value, ctypes.byref(n)))
    return out[:n.value]


def alpa_dp_best(h) -> dict:
    plan = alpa_plan_t()
    _check(load().alpa_dp_best(h, ctypes.byref(plan)))
    return plan.as_dict()


def alpa_dp_last_timing(h):
    a, b, c = ctypes.c_float(), ctypes.c_float(), ctypes.c_float()
    _check(load().alpa_dp_last_timing(h, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)))
    return dict(ms_candidates=a.value, ms_recurrence=b.value, ms_epilogue=c.value)


def alpa_dp_last_counters(h):
    n, w = ctypes.c_int(), ctypes.c_int64()
    _check(load().alpa_dp_last_counters(h, ctypes.byref(n), ctypes.byref(w)))
    return dict(n_candidates=n.value, wave_relaxations=w.value)


def alpa_dp_destroy(h):
    load().alpa_dp_destroy(h)


def plan_from_bytes(buf: bytes) -> dict:
    return alpa_plan_t.from_buffer_copy(buf).as_dict()


PLAN_BYTES = ctypes.sizeof(alpa_plan_t)


def alpa_cluster_layers_exact(flop, edge_src, edge_dst, edge_bytes, L, delta_ppm):
    """Operator clustering with the variance tie-break taken over whole clusterings."""
    return alpa_cluster_layers(flop, edge_src, edge_dst, edge_bytes, L, delta_ppm,
                               _fn="alpa_cluster_layers_exact")


def alpa_cluster_layers(flop, edge_src, edge_dst, edge_bytes, L, delta_ppm,
                        _fn="alpa_cluster_layers"):
    """Operator clustering (Eq. 6).  Host arrays in; returns dict(comm, sumsq, first_op, ms);
    comm == INF_I64 and first_op == [] if no clustering satisfies the FLOP bound."""
    lib = load()
    f = np.ascontiguousarray(flop, dtype=np.int32)
    s = np.ascontiguousarray(edge_src, dtype=np.int32)
    d = np.ascontiguousarray(edge_dst, dtype=np.int32)
    b = np.ascontiguousarray(edge_bytes, dtype=np.int64)
    if not (s.size == d.size == b.size):
        raise ValueError("edge arrays must have one length")
    comm, sumsq, ms = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_float()
    first = np.zeros(max(int(L), 0) + 1, dtype=np.int32)
    _check(getattr(lib, _fn)(f.ctypes.data, int(f.size), s.ctypes.data if s.size else None,
                                   d.ctypes.data if s.size else None,
                                   b.ctypes.data if s.size else None, int(s.size), int(L),
                                   int(delta_ppm), ctypes.byref(comm), ctypes.byref(sumsq),
                                   first.ctypes.data, ctypes.byref(ms)))
    feasible = comm.value != INF_I64
    return {"comm": int(comm.value), "sumsq": int(sumsq.value),
            "first_op": [int(x) for x in first] if feasible else [], "ms": float(ms.value)}


def alpa_cluster_layers_static(d_flop, d_edge_src, d_edge_dst, d_edge_bytes, L, delta_ppm, d_out,
                               d_out_first_op, stream=None):
    """Allocation-free, asynchronous variant: torch CUDA tensors in (int32 / int32 / int32 /
    int64) and out (d_out int64 [3], d_out_first_op int32 [L + 1]); stream: a torch.cuda.Stream,
    a raw handle or None (null stream)."""
    def ptr(t):
        return None if t is None or t.numel() == 0 else ctypes.c_void_p(int(t.data_ptr()))
    raw = 0 if stream is None else int(getattr(stream, "cuda_stream", stream))
    E = 0 if d_edge_src is None else int(d_edge_src.numel())
    _check(load().alpa_cluster_layers_static(ptr(d_flop), int(d_flop.numel()), ptr(d_edge_src),
                                             ptr(d_edge_dst), ptr(d_edge_bytes), E, int(L),
                                             int(delta_ppm), ptr(d_out), ptr(d_out_first_op),
                                             ctypes.c_void_p(raw)))


def alpa_place_submeshes(N, M, stage_shapes):
    """stage_shapes: (n, m) per stage in pipeline order.  Returns [(row, col)] per stage."""
    shp = np.ascontiguousarray(stage_shapes, dtype=np.int32).reshape(-1, 2)
    n = shp.shape[0]
    arr = (alpa_shape_t * max(n, 1))(*[alpa_shape_t(int(a), int(b)) for a, b in shp])
    row = np.zeros(max(n, 1), np.int32)
    col = np.zeros(max(n, 1), np.int32)
    _check(load().alpa_place_submeshes(int(N), int(M), arr, n, row.ctypes.data, col.ctypes.data))
    return [(int(r), int(c)) for r, c in zip(row[:n], col[:n])]


def alpa_dp_measure_valu_peak() -> float:
    """Sustained int32 add + min rate of the current device, lane-operations per second."""
    out = ctypes.c_double()
    _check(load().alpa_dp_measure_valu_peak(ctypes.byref(out)))
    return float(out.value)
