"""GPU parity of the table construction step (Sec. 5.2, Eq. 5, Alg. 1's intra-op loop nest):
the table the library builds on the device against the oracle's, bit-exact, and the dynamic
program on top of it."""
import ctypes
import hashlib
import json
import os

import numpy as np
import pytest

import oracle
from paper_2201_12023_amd import binding as B
from paper_2201_12023_amd import workloads as W
from tests.table_cases import INF32, load_example

pytestmark = pytest.mark.gpu

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _device_table(p, K, N, M, shapes, Bm=4):
    h = B.alpa_dp_create_from_profiles(p[0], p[1], p[2], p[3], K, N, M, Bm, shapes)
    try:
        return B.alpa_dp_get_table(h, K, len(shapes)), B.alpa_dp_count_candidates(h)
    finally:
        B.alpa_dp_destroy(h)


def test_hand_worked_example_on_the_device():
    t_l, ms, ma, dev, exp = load_example()
    got, n = _device_table((t_l, ms, ma, dev), 3, 1, 1, np.asarray([[1, 1]], np.int32))
    assert (got == exp).all()
    assert n == len(np.unique(exp[exp != INF32]))


RANDOM = [  # seed, K, N, M, O
    (0, 1, 1, 1, 1), (1, 2, 1, 2, 3), (2, 5, 2, 2, 2), (3, 9, 3, 4, 7), (4, 17, 1, 8, 4),
    (5, 33, 2, 4, 5), (6, 64, 8, 8, 6), (7, 23, 4, 2, 32), (8, 70, 3, 8, 3), (9, 12, 16, 8, 9),
]


@pytest.mark.parametrize("case", RANDOM, ids=lambda c: f"s{c[0]}-K{c[1]}-{c[2]}x{c[3]}-O{c[4]}")
def test_random_profiles(case):
    """Unstructured figures: ties, absent options, zero activation sizes; sizes from one thread
    to several blocks with a ragged tail, up to the maximum number of options."""
    seed, K, N, M, O = case
    shapes = W.submesh_shapes(N, M)
    p = W.random_profiles(seed, K, len(shapes), O, absent_frac=[0.0, 0.2, 0.7][seed % 3])
    ref = oracle.build_table(p.t_l, p.mem_stage, p.mem_act, p.mem_device)
    got, n = _device_table((p.t_l, p.mem_stage, p.mem_act, p.mem_device), K, N, M, shapes)
    assert (got == ref).all()
    assert n == len(oracle.all_candidates(ref, shapes))


@pytest.mark.parametrize("idx", [1, 2, 3, 4, 5])
def test_workload_profiles_table_and_dp_on_top(idx):
    """Six options per (stage, submesh) at the workloads' real sizes; then the dynamic program
    on the device-built table against the oracle on the oracle-built table."""
    w = W.make_workload(idx)
    p = W.make_profiles(idx, 6)
    ref = oracle.build_table(p.t_l, p.mem_stage, p.mem_act, p.mem_device)
    h = B.alpa_dp_create_from_profiles(p.t_l, p.mem_stage, p.mem_act, p.mem_device, w.K, w.N,
                                       w.M, w.B, w.shapes)
    try:
        assert (B.alpa_dp_get_table(h, w.K, w.S) == ref).all()
        allc = oracle.all_candidates(ref, w.shapes)
        assert B.alpa_dp_count_candidates(h) == len(allc)
        cand = oracle.quantiles(allc, 24)
        T_ref, p_ref = oracle.solve_parallel(ref, w.N, w.M, w.B, w.shapes, cand, False, 8)
        T, plan = B.alpa_dp_solve(h, None, 24, 0)
        assert (B.alpa_dp_candidates(h) == cand).all()
        assert (T == T_ref).all()
        assert plan["T_star"] == p_ref.T_star and plan["t_max"] == p_ref.t_max
        assert plan["first_layer"] == p_ref.first_layer and plan["shape_idx"] == p_ref.shape_idx
    finally:
        B.alpa_dp_destroy(h)


def test_deep_model_profiles_table_and_dp_on_top():
    """100 layers on a 4x8 mesh: the table built on the device feeds the 7-wave form of the
    register/LDS kernel."""
    K, N, M, Bm = 100, 4, 8, 16
    shapes = W.submesh_shapes(N, M)
    p = W.random_profiles(21, K, len(shapes), 3, absent_frac=0.2)
    ref = oracle.build_table(p.t_l, p.mem_stage, p.mem_act, p.mem_device)
    h = B.alpa_dp_create_from_profiles(p.t_l, p.mem_stage, p.mem_act, p.mem_device, K, N, M, Bm,
                                       shapes)
    try:
        assert (B.alpa_dp_get_table(h, K, len(shapes)) == ref).all()
        cand = oracle.quantiles(oracle.all_candidates(ref, shapes), 24)
        T_ref, p_ref = oracle.solve_parallel(ref, N, M, Bm, shapes, cand, False, 8)
        T, plan = B.alpa_dp_solve(h, None, 24, 0)
        assert (B.alpa_dp_candidates(h) == cand).all()
        assert (T == T_ref).all()
        assert plan["T_star"] == p_ref.T_star and plan["t_max"] == p_ref.t_max
        assert plan["first_layer"] == p_ref.first_layer and plan["shape_idx"] == p_ref.shape_idx
    finally:
        B.alpa_dp_destroy(h)


@pytest.mark.parametrize("idx", [2, 4])
def test_single_option_profiles_give_the_workload_table(idx):
    w = W.make_workload(idx)
    p = W.single_option_profiles(w)
    got, n = _device_table((p.t_l, p.mem_stage, p.mem_act, p.mem_device), w.K, w.N, w.M, w.shapes)
    assert (got == w.table).all()
    g = json.load(open(os.path.join(GOLD, f"workload_{idx}.json")))
    assert hashlib.sha256(got.tobytes()).hexdigest() == g["table_sha256"]
    assert n == g["n_distinct"]


def test_nothing_fits_and_everything_absent():
    shapes = W.submesh_shapes(2, 2)
    p = W.random_profiles(3, 6, len(shapes), 4)
    got, n = _device_table((p.t_l, p.mem_stage + 1, p.mem_act, 0), 6, 2, 2, shapes)
    assert (got == INF32).all() and n == 0
    t_l = np.full_like(p.t_l, INF32)
    got, n = _device_table((t_l, p.mem_stage, p.mem_act, p.mem_device), 6, 2, 2, shapes)
    assert (got == INF32).all() and n == 0


def test_argument_errors():
    L = B.load()
    K, N, M = 4, 2, 2
    shapes = W.submesh_shapes(N, M)
    S = len(shapes)
    arr = (B.alpa_shape_t * S)(*[B.alpa_shape_t(int(n), int(m)) for n, m in shapes])
    p = W.random_profiles(1, K, S, 3)

    def rc(t_l=p.t_l, ms=p.mem_stage, ma=p.mem_act, O=3, dev=p.mem_device, K_=K):
        h = ctypes.c_void_p()
        r = L.alpa_dp_create_from_profiles(
            ctypes.byref(h), t_l.ctypes.data if t_l is not None else None,
            ms.ctypes.data if ms is not None else None,
            ma.ctypes.data if ma is not None else None, O, dev, K_, N, M, 2, arr, S)
        if r == 0:
            L.alpa_dp_destroy(h)
        else:
            assert h.value is None
        return r

    assert rc() == 0
    assert rc(t_l=None) == -1 and rc(ms=None) == -1 and rc(ma=None) == -1
    assert rc(O=0) == -1 and rc(O=B.MAX_OPTIONS + 1) == -1
    assert rc(dev=-1) == -1 and rc(K_=0) == -1
    bad = p.t_l.copy(); bad[0, 1, 0, 0] = -3
    assert rc(t_l=bad) == -1
    bad = p.mem_stage.copy(); bad[1, 2, 1, 2] = -1
    assert rc(ms=bad) == -1
    bad = p.mem_act.copy(); bad[0, 0, 0, 0] = 2**52
    assert rc(ma=bad) == -1
    # figures below the diagonal are not looked at
    ok = p.mem_act.copy(); ok[2, 0, 0, 0] = -9
    assert rc(ma=ok) == 0
    # the overflow proof is made on the table that results, not on options that never fit
    big = p.t_l.copy(); big[0, 0, 0, 0] = 2**30 // K; big[0, 0, 0, 1:] = INF32
    ms2 = p.mem_stage.copy(); ms2[0, 0, 0, 0] = p.mem_device + 1
    assert rc(t_l=big, ms=ms2) == 0
    ms2[0, 0, 0, 0] = 0
    ma2 = p.mem_act.copy(); ma2[0, 0, 0, 0] = 0
    assert rc(t_l=big, ms=ms2, ma=ma2) == -2
    assert L.alpa_dp_get_table(None, None) == -1
