"""GPU parity: the HIP library (through the C ABI) against the CPU oracle, bit-exact."""
import hashlib
import json
import os

import numpy as np
import pytest

import oracle
from paper_2201_12023_amd import binding as B
from paper_2201_12023_amd import workloads as W

pytestmark = pytest.mark.gpu

INF64 = oracle.INF64
GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
KERNELS = {"fast": 0, "generic": B.ALPA_DP_GENERIC}


def _same_plan(gpu: dict, ref: oracle.Plan):
    assert gpu["T_star"] == ref.T_star
    assert gpu["t_max"] == ref.t_max
    assert gpu["num_stages"] == ref.num_stages
    assert gpu["n_evaluated"] == ref.n_evaluated
    assert gpu["first_layer"] == ref.first_layer
    assert gpu["shape_idx"] == ref.shape_idx


def _full_check(w, kernel_flag, prune):
    """Every candidate's T*, the candidate list itself, and the plan, against the oracle."""
    cand_ref = oracle.all_candidates(w.table, w.shapes)
    T_ref, p_ref = oracle.solve(w.table, w.N, w.M, w.B, w.shapes, cand_ref, prune)
    h = B.alpa_dp_create(w.table, w.K, w.N, w.M, w.B, w.shapes)
    try:
        assert B.alpa_dp_count_candidates(h) == len(cand_ref)
        flags = kernel_flag | (B.ALPA_DP_PRUNE if prune else 0)
        T, plan = B.alpa_dp_solve(h, None, 0, flags)
        cand = B.alpa_dp_candidates(h)
        assert (cand == cand_ref).all()
        assert (T == T_ref).all()
        _same_plan(plan, p_ref)
        _same_plan(B.alpa_dp_best(h), p_ref)
    finally:
        B.alpa_dp_destroy(h)


@pytest.mark.parametrize("kernel", list(KERNELS))
@pytest.mark.parametrize("prune", [False, True])
@pytest.mark.parametrize("idx", [1, 2])
def test_small_workloads_all_candidates(idx, prune, kernel):
    _full_check(W.make_workload(idx), KERNELS[kernel], prune)


RANDOM_CASES = [
    # seed, K, N, M
    (0, 1, 1, 1), (1, 2, 1, 2), (2, 3, 2, 2), (3, 5, 1, 4), (4, 6, 2, 4), (5, 7, 3, 2),
    (6, 9, 3, 4), (7, 12, 2, 8), (8, 17, 4, 4), (9, 16, 1, 8), (10, 33, 2, 2), (11, 20, 5, 4),
    (12, 10, 8, 8), (13, 40, 3, 8), (14, 64, 1, 2), (15, 13, 7, 8),
    # more shapes than the register/LDS kernel's early-stop table covers (18, then the maximum 64)
    (16, 30, 16, 4), (17, 20, 64, 1), (18, 64, 5, 8), (19, 57, 8, 8),
]


@pytest.mark.parametrize("kernel", list(KERNELS))
@pytest.mark.parametrize("case", RANDOM_CASES, ids=lambda c: f"s{c[0]}-K{c[1]}-{c[2]}x{c[3]}")
def test_random_tables(case, kernel):
    """Unstructured tables (not monotone in stage length), many infinities and ties; sizes
    span one to four 16-layer blocks, ragged tails, non-power-of-two device counts."""
    seed, K, N, M = case
    rng = np.random.default_rng(seed)
    w = W.random_problem(seed, K, N, M, inf_frac=float(rng.choice([0.0, 0.2, 0.6])),
                         value_hi=int(rng.choice([4, 50, 5000])))
    cand_ref = oracle.all_candidates(w.table, w.shapes)
    if len(cand_ref) > 300:            # keep the oracle's share of the test short
        cand_ref = oracle.quantiles(cand_ref, 300)
    for prune in (False, True):
        T_ref, p_ref = oracle.solve_parallel(w.table, w.N, w.M, w.B, w.shapes, cand_ref, prune, 8)
        h = B.alpa_dp_create(w.table, w.K, w.N, w.M, w.B, w.shapes)
        try:
            flags = KERNELS[kernel] | (B.ALPA_DP_PRUNE if prune else 0)
            # an empty list is an argument error at the boundary; an all-infinite table is
            # reached through the "candidates from the table" mode instead
            T, plan = B.alpa_dp_solve(h, cand_ref if len(cand_ref) else None, flags=flags)
            assert (T == T_ref).all()
            _same_plan(plan, p_ref)
        finally:
            B.alpa_dp_destroy(h)


def test_caller_order_duplicates_and_out_of_table_values():
    w = W.make_workload(2)
    allc = oracle.all_candidates(w.table, w.shapes)
    rng = np.random.default_rng(5)
    mine = np.concatenate([rng.choice(allc, 200), rng.choice(allc, 50), [0, 1, 2**31 - 2, 7, 7],
                           allc[-3:]]).astype(np.int32)
    rng.shuffle(mine)
    uniq = oracle.sort_dedup(mine)
    for prune in (False, True):
        T_ref, p_ref = oracle.solve(w.table, w.N, w.M, w.B, w.shapes, uniq, prune)
        h = B.alpa_dp_create(w.table, w.K, w.N, w.M, w.B, w.shapes)
        try:
            T, plan = B.alpa_dp_solve(h, mine, flags=B.ALPA_DP_PRUNE if prune else 0)
            assert (B.alpa_dp_candidates(h) == uniq).all()
            pos = np.searchsorted(uniq, mine)
            assert (T == T_ref[pos]).all()
            _same_plan(plan, p_ref)
        finally:
            B.alpa_dp_destroy(h)


def test_quantile_mode_and_errors():
    w = W.make_workload(2)
    allc = oracle.all_candidates(w.table, w.shapes)
    h = B.alpa_dp_create(w.table, w.K, w.N, w.M, w.B, w.shapes)
    try:
        for Q in (2, 3, 64, 257, len(allc), len(allc) + 5):
            cand = oracle.quantiles(allc, Q)
            T_ref, p_ref = oracle.solve(w.table, w.N, w.M, w.B, w.shapes, cand, False)
            T, plan = B.alpa_dp_solve(h, None, Q, 0)
            assert (B.alpa_dp_candidates(h) == cand).all()
            assert (T == T_ref).all()
            _same_plan(plan, p_ref)
        L = B.load()
        assert L.alpa_dp_solve(h, None, 1, 0, None, None) == -1
        assert L.alpa_dp_solve(h, None, -1, 0, None, None) == -1
        bad = np.asarray([5, -1], np.int32)
        assert L.alpa_dp_solve(h, bad.ctypes.data, 2, 0, None, None) == -1
        bad = np.asarray([5, 2**31 - 1], np.int32)
        assert L.alpa_dp_solve(h, bad.ctypes.data, 2, 0, None, None) == -1
        assert L.alpa_dp_solve(h, bad.ctypes.data, 0, 0, None, None) == -1
    finally:
        B.alpa_dp_destroy(h)


def test_infeasible_and_degenerate_problems():
    # every entry infinite
    w = W.random_problem(1, 4, 2, 2, inf_frac=1.0)
    h = B.alpa_dp_create(w.table, w.K, w.N, w.M, w.B, w.shapes)
    try:
        assert B.alpa_dp_count_candidates(h) == 0
        T, plan = B.alpa_dp_solve(h, None, 0, 0)
        assert len(T) == 0 and plan["T_star"] == INF64 and plan["num_stages"] == 0
        T, plan = B.alpa_dp_solve(h, [3, 9], flags=B.ALPA_DP_PRUNE)
        assert (T == INF64).all() and plan["T_star"] == INF64 and plan["n_evaluated"] == 2
    finally:
        B.alpa_dp_destroy(h)
    # more devices than layers with one-device submeshes only: no plan
    shapes = np.asarray([[1, 1]], np.int32)
    table = np.full((3, 3, 3, 1), 5, np.int32)
    h = B.alpa_dp_create(table, 3, 4, 1, 2, shapes)
    try:
        T, plan = B.alpa_dp_solve(h, None, 0, 0)
        assert (T == INF64).all() and plan["num_stages"] == 0
    finally:
        B.alpa_dp_destroy(h)
    # a candidate below every entry
    w = W.make_workload(1)
    h = B.alpa_dp_create(w.table, w.K, w.N, w.M, w.B, w.shapes)
    try:
        T, plan = B.alpa_dp_solve(h, [0, 1])
        assert (T == INF64).all() and plan["T_star"] == INF64
    finally:
        B.alpa_dp_destroy(h)


def test_prune_breaks_on_equality_gpu():
    K, Bm = 2, 2
    shapes = np.asarray([[1, 1], [2, 1]], np.int32)
    table = np.full((K, K, K, 2), 2**31 - 1, np.int64)
    table[:, 0, 0, 0] = 2
    table[:, 1, 1, 0] = 2
    table[:, 0, 1, 1] = 3
    table = table.astype(np.int32)
    for kf in KERNELS.values():
        h = B.alpa_dp_create(table, K, 2, 1, Bm, shapes)
        try:
            T, plan = B.alpa_dp_solve(h, None, 0, kf | B.ALPA_DP_PRUNE)
            assert list(T) == [6, INF64] and plan["n_evaluated"] == 1 and plan["t_max"] == 2
            T, plan = B.alpa_dp_solve(h, None, 0, kf)
            assert list(T) == [6, 6] and plan["n_evaluated"] == 2 and plan["t_max"] == 2
        finally:
            B.alpa_dp_destroy(h)


def test_best_over_several_solves_and_set_B():
    w = W.make_workload(2)
    allc = oracle.all_candidates(w.table, w.shapes)
    h = B.alpa_dp_create(w.table, w.K, w.N, w.M, w.B, w.shapes)
    try:
        lo, hi = allc[: len(allc) // 3], allc[len(allc) // 3:]
        _, p_hi = oracle.solve(w.table, w.N, w.M, w.B, w.shapes, hi, False)
        _, p_lo = oracle.solve(w.table, w.N, w.M, w.B, w.shapes, lo, False)
        _, g_hi = B.alpa_dp_solve(h, hi)
        _same_plan(g_hi, p_hi)
        _, g_lo = B.alpa_dp_solve(h, lo)
        _same_plan(g_lo, p_lo)
        best = B.alpa_dp_best(h)
        ref = min([p_hi, p_lo], key=lambda p: (p.T_star, p.t_max))
        _same_plan(best, ref)
        # another B: Eq. 4 and the pruning rule change, F does not
        B.alpa_dp_set_B(h, 3)
        T_ref, p_ref = oracle.solve(w.table, w.N, w.M, 3, w.shapes, allc, True)
        T, plan = B.alpa_dp_solve(h, None, 0, B.ALPA_DP_PRUNE)
        assert (T == T_ref).all()
        _same_plan(plan, p_ref)
        # T* under B = 32 and under B = 3 do not compare: the running best started over with
        # the new B (the old one, found with the larger B, has the larger T*)
        _same_plan(B.alpa_dp_best(h), p_ref)
        B.alpa_dp_set_B(h, 3)                      # no change of B: the best stays
        _same_plan(B.alpa_dp_best(h), p_ref)
        # back to a larger B with no solve since: alpa_dp_best runs the pruned loop itself
        B.alpa_dp_set_B(h, 50)
        _, p50 = oracle.solve(w.table, w.N, w.M, 50, w.shapes, allc, True)
        _same_plan(B.alpa_dp_best(h), p50)
    finally:
        B.alpa_dp_destroy(h)
    # alpa_dp_best on a fresh handle runs the full pruned loop itself
    h = B.alpa_dp_create(w.table, w.K, w.N, w.M, w.B, w.shapes)
    try:
        _, p_ref = oracle.solve(w.table, w.N, w.M, w.B, w.shapes, allc, True)
        _same_plan(B.alpa_dp_best(h), p_ref)
    finally:
        B.alpa_dp_destroy(h)


def test_best_after_a_sweep_only_runs_the_pruned_loop():
    """A sweep leaves the running best alone, so alpa_dp_best on a handle that has only seen
    a sweep (or nothing since its table was restricted) still runs Alg. 1's loop itself."""
    w = W.make_workload(2)
    allc = oracle.all_candidates(w.table, w.shapes)
    _, p_ref = oracle.solve(w.table, w.N, w.M, w.B, w.shapes, allc, True)
    h = B.alpa_dp_create(w.table, w.K, w.N, w.M, w.B, w.shapes)
    try:
        plans = B.alpa_dp_solve_sweep(h, None, [2, 7])
        assert plans[0]["num_stages"] > 0
        assert len(B.alpa_dp_candidates(h)) == len(allc)      # the sweep counts as a solve here
        _same_plan(B.alpa_dp_best(h), p_ref)
        B.alpa_dp_solve_sweep(h, None, [5])
        _same_plan(B.alpa_dp_best(h), p_ref)
    finally:
        B.alpa_dp_destroy(h)


def test_candidates_from_two_to_the_thirty_on_are_no_filter():
    """Host candidates may be as large as INT32_MAX - 1; from the device's +infinity sentinel
    (2^30 - 1) on they filter nothing, and Eq. 4 still adds (B - 1) times the value given."""
    w = W.make_workload(2)
    big = np.array([(1 << 30) - 2, (1 << 30) - 1, 1 << 30, 0x3f3f3f3f, 0x3f3f3f40, (1 << 31) - 2,
                    1000, 1500], dtype=np.int32)
    for kernel in KERNELS.values():
        for nc in (1, 2):
            T_ref, p_ref = oracle.solve(w.table, w.N, w.M, w.B, w.shapes, np.unique(big), False)
            by_value = dict(zip(np.unique(big).tolist(), T_ref.tolist()))
            h = B.alpa_dp_create(w.table, w.K, w.N, w.M, w.B, w.shapes)
            try:
                B.alpa_dp_set_tuning(h, B.ALPA_DP_TUNE_CANDIDATES_PER_WG, nc)
                T, plan = B.alpa_dp_solve(h, big, flags=kernel)
                assert T.tolist() == [by_value[int(c)] for c in big]
                _same_plan(plan, p_ref)
            finally:
                B.alpa_dp_destroy(h)


def test_create_checks_the_range_of_the_table_on_the_device():
    import ctypes
    w = W.make_workload(1)
    L = B.load()
    arr = (B.alpa_shape_t * w.S)(*[B.alpa_shape_t(int(n), int(m)) for n, m in w.shapes])

    def create_rc(table):
        h = ctypes.c_void_p()
        rc = L.alpa_dp_create(ctypes.byref(h), table.ctypes.data, w.K, w.N, w.M, w.B, arr, w.S)
        assert (h.value is None) == (rc != 0)
        if rc == 0:
            L.alpa_dp_destroy(h)
        return rc, L.alpa_dp_last_error().decode()

    for pos in ((0, 0, 0, 0), (w.K - 1, w.K - 1, w.K - 1, w.S - 1), (2, 1, 5, 1)):
        neg = w.table.copy(); neg[pos] = -5
        rc, msg = create_rc(neg)
        assert rc == -1 and "negative" in msg
    # entries below the diagonal are not part of the problem and are not checked
    low = w.table.copy(); low[0, 3, 1, 0] = -7; low[1, 4, 0, 2] = 2**30
    assert create_rc(low)[0] == 0
    big = w.table.copy(); big[big != W.INF_I32] = 2**30 // w.K
    rc, msg = create_rc(big)
    assert rc == -2 and "2^30" in msg
    ok = w.table.copy(); ok[ok != W.INF_I32] = (2**30 - 1) // w.K
    assert create_rc(ok)[0] == 0
    allinf = np.full_like(w.table, W.INF_I32)
    assert create_rc(allinf)[0] == 0


LANE_GROUP_CASES = [  # seed, K, N, M: every group width 1, 2, 4, 8, 16, 32 and meshes that do
    # not fill their group (3, 6, 10, 12, 24 devices)
    (700, 9, 1, 1), (701, 20, 1, 2), (702, 14, 3, 1), (703, 33, 1, 4), (704, 25, 3, 2),
    (705, 48, 1, 8), (706, 17, 5, 2), (707, 30, 3, 4), (708, 64, 2, 8), (709, 40, 3, 8),
    (710, 22, 1, 32), (711, 64, 4, 8), (712, 100, 2, 16), (713, 70, 1, 4), (714, 5, 2, 16),
]


@pytest.mark.parametrize("prune", [False, True])
@pytest.mark.parametrize("case", LANE_GROUP_CASES, ids=lambda c: f"s{c[0]}-K{c[1]}-{c[2]}x{c[3]}")
def test_small_meshes_in_lane_groups(case, prune):
    """On meshes of up to 32 devices the register/LDS kernel cuts the wave into groups of lanes
    with a candidate each (64, 32, ... 2 candidates per workgroup).  Unstructured tables with a
    narrow value range (neighbouring candidates then differ in few entries: the lane-by-lane
    filter) and formula tables; every candidate, quantiles, and an unsorted caller list with
    repeats whose length is no multiple of the group count; against the oracle, and against
    the same kernel with the groups switched off."""
    seed, K, N, M = case
    rng = np.random.default_rng(seed)
    if seed % 3 == 2:
        w = W.deep_model_problem(seed, K, N, M)
    else:
        w = W.random_problem(seed, K, N, M, inf_frac=float(rng.choice([0.0, 0.2, 0.5])),
                             value_hi=int(rng.choice([5, 60, 5000])))
    allc = oracle.all_candidates(w.table, w.shapes)
    if len(allc) == 0:
        pytest.skip("no finite entry")
    lists = [allc if len(allc) <= 400 else oracle.quantiles(allc, 397)]
    hi = int(allc[-1]) + 3
    lists.append(rng.integers(0, hi, size=int(rng.integers(1, 150))).astype(np.int32))
    flags = B.ALPA_DP_PRUNE if prune else 0
    h = B.alpa_dp_create(w.table, w.K, w.N, w.M, w.B, w.shapes)
    try:
        for cand in lists:
            srt = np.unique(cand)
            T_ref, p_ref = oracle.solve_parallel(w.table, w.N, w.M, w.B, w.shapes, srt, prune, 8)
            by_value = dict(zip(srt.tolist(), T_ref.tolist()))
            for groups in (64, 2):                  # as many as the mesh allows; two
                B.alpa_dp_set_tuning(h, B.ALPA_DP_TUNE_LANE_GROUPS, groups)
                T, plan = B.alpa_dp_solve(h, cand, flags=flags)
                assert T.tolist() == [by_value[int(c)] for c in cand]
                _same_plan(plan, p_ref)
            B.alpa_dp_set_tuning(h, B.ALPA_DP_TUNE_LANE_GROUPS, 1)
            T1, plan1 = B.alpa_dp_solve(h, cand, flags=flags)
            assert (T1 == T).all() and plan1 == plan
        # no list: the table's own values, all of them, with the library's own choice of groups
        B.alpa_dp_set_tuning(h, B.ALPA_DP_TUNE_LANE_GROUPS, 0)
        T_ref, p_ref = oracle.solve_parallel(w.table, w.N, w.M, w.B, w.shapes, allc, prune, 8)
        T, plan = B.alpa_dp_solve(h, None, 0, flags)
        assert (T == T_ref).all()
        _same_plan(plan, p_ref)
        plans = B.alpa_dp_solve_sweep(h, None, [1, 3, w.B], flags=flags)
        for Bv, pl in zip([1, 3, w.B], plans):
            _, pb = oracle.solve_parallel(w.table, w.N, w.M, Bv, w.shapes, allc, prune, 8)
            _same_plan(pl, pb)
    finally:
        B.alpa_dp_destroy(h)


def test_tuning_call_rejects_what_it_does_not_know():
    w = W.make_workload(1)
    L = B.load()
    h = B.alpa_dp_create(w.table, w.K, w.N, w.M, w.B, w.shapes)
    try:
        assert L.alpa_dp_set_tuning(None, 1, 1) == -1
        assert L.alpa_dp_set_tuning(h, 99, 1) == -1
        assert L.alpa_dp_set_tuning(h, B.ALPA_DP_TUNE_CANDIDATES_PER_WG, 3) == -1
        assert L.alpa_dp_set_tuning(h, B.ALPA_DP_TUNE_DISTINCT_BY_SORT, 2) == -1
        assert L.alpa_dp_set_tuning(h, B.ALPA_DP_TUNE_WG_PER_CU, -1) == -1
        assert L.alpa_dp_set_tuning(h, B.ALPA_DP_TUNE_LANE_GROUPS, 3) == -1
        assert L.alpa_dp_set_tuning(h, B.ALPA_DP_TUNE_LANE_GROUPS, 128) == -1
        assert L.alpa_dp_set_tuning(h, B.ALPA_DP_TUNE_WORKGROUPS, -1) == -1
        ref = oracle.all_candidates(w.table, w.shapes)
        T_ref, p_ref = oracle.solve(w.table, w.N, w.M, w.B, w.shapes, ref, False)
        for key, value in ((B.ALPA_DP_TUNE_WG_PER_CU, 1), (B.ALPA_DP_TUNE_WG_PER_CU, 0),
                           (B.ALPA_DP_TUNE_DISTINCT_BY_SORT, 1), (B.ALPA_DP_TUNE_DISTINCT_BY_SORT, 0)):
            B.alpa_dp_set_tuning(h, key, value)
            T, plan = B.alpa_dp_solve(h, None, 0, 0)
            assert (T == T_ref).all()
            _same_plan(plan, p_ref)
    finally:
        B.alpa_dp_destroy(h)


def test_device_pointer_variant_on_a_torch_stream():
    import torch
    w = W.make_workload(2)
    allc = oracle.all_candidates(w.table, w.shapes)
    cand = oracle.quantiles(allc, 500)
    T_ref, p_ref = oracle.solve(w.table, w.N, w.M, w.B, w.shapes, cand, False)
    st = torch.cuda.Stream()
    h = B.alpa_dp_create(w.table, w.K, w.N, w.M, w.B, w.shapes)
    try:
        B.alpa_dp_set_stream(h, st)
        with torch.cuda.stream(st):
            d_t = torch.from_numpy(cand[::-1].copy()).to("cuda", non_blocking=False)
            d_T = torch.empty(len(cand), dtype=torch.int64, device="cuda")
            d_plan = torch.zeros(B.PLAN_BYTES, dtype=torch.uint8, device="cuda")
        st.synchronize()
        for _ in range(3):
            B.alpa_dp_solve_dev(h, d_t, len(cand), 0, d_T, d_plan)
        st.synchronize()
        assert (d_T.cpu().numpy()[::-1] == T_ref).all()
        _same_plan(B.plan_from_bytes(d_plan.cpu().numpy().tobytes()), p_ref)
        tm = B.alpa_dp_last_timing(h)
        assert tm["ms_recurrence"] > 0
    finally:
        B.alpa_dp_destroy(h)


@pytest.mark.parametrize("idx", [3, 4, 5])
def test_full_size_workloads_against_stored_oracle_results(idx):
    """Workloads 3-5 at full size in the launch configuration the benchmark times.  The
    expected values were written by tests/golden/make_golden.py from the oracle alone."""
    g = json.load(open(os.path.join(GOLD, f"workload_{idx}.json")))
    w = W.make_workload(idx)
    assert hashlib.sha256(w.table.tobytes()).hexdigest() == g["table_sha256"]
    h = B.alpa_dp_create(w.table, w.K, w.N, w.M, w.B, w.shapes)
    try:
        assert B.alpa_dp_count_candidates(h) == g["n_distinct"]
        nq = w.n_quantiles if w.candidates == "quantiles" else 0
        T, plan = B.alpa_dp_solve(h, None, nq, B.ALPA_DP_PRUNE if w.prune else 0)
        cand = B.alpa_dp_candidates(h)
        assert len(cand) == g["n_candidates"]
        assert hashlib.sha256(cand.astype("<i4").tobytes()).hexdigest() == g["cand_sha256"]
        assert [int(x) for x in T[::97]] == g["T_every_97"]
        assert hashlib.sha256(T.astype("<i8").tobytes()).hexdigest() == g["T_sha256"]
        for key in ("T_star", "t_max", "num_stages", "n_evaluated", "first_layer", "shape_idx"):
            assert plan[key] == g["plan"][key], key
        # a few candidates recomputed by the oracle now, one by one
        pick = np.linspace(0, len(cand) - 1, 6).astype(int)
        T_o, _ = oracle.eval_candidates(w.table, w.N, w.M, w.B, w.shapes, cand[pick], threads=6)
        assert (T[pick] == T_o).all()
    finally:
        B.alpa_dp_destroy(h)


def test_general_kernel_on_a_mesh_larger_than_64_devices():
    """N*M = 80 and K = 66 are outside the register/LDS kernel; the general one serves."""
    w = W.random_problem(77, 66, 10, 8, inf_frac=0.3, value_hi=900)
    allc = oracle.all_candidates(w.table, w.shapes)
    cand = oracle.quantiles(allc, 8)
    T_ref, p_ref = oracle.solve_parallel(w.table, w.N, w.M, w.B, w.shapes, cand, False, 8)
    h = B.alpa_dp_create(w.table, w.K, w.N, w.M, w.B, w.shapes)
    try:
        T, plan = B.alpa_dp_solve(h, cand)
        assert (T == T_ref).all()
        _same_plan(plan, p_ref)
    finally:
        B.alpa_dp_destroy(h)


@pytest.mark.parametrize("case", [(91, 256, 1, 2), (92, 5, 32, 32), (93, 40, 16, 16)],
                         ids=["K256-1x2", "K5-32x32", "K40-16x16"])
def test_general_kernel_at_the_size_limits(case):
    """The largest K (256), the largest mesh (1024 devices, 37 shapes) and one in between."""
    seed, K, N, M = case
    w = W.random_problem(seed, K, N, M, inf_frac=0.2, value_hi=3000)
    cand = oracle.quantiles(oracle.all_candidates(w.table, w.shapes), 6)
    for prune in (False, True):
        T_ref, p_ref = oracle.solve_parallel(w.table, w.N, w.M, w.B, w.shapes, cand, prune, 6)
        h = B.alpa_dp_create(w.table, w.K, w.N, w.M, w.B, w.shapes)
        try:
            T, plan = B.alpa_dp_solve(h, cand, flags=B.ALPA_DP_PRUNE if prune else 0)
            assert (T == T_ref).all()
            _same_plan(plan, p_ref)
        finally:
            B.alpa_dp_destroy(h)


def test_valu_peak_probe_and_readme_example():
    rate = B.alpa_dp_measure_valu_peak()
    assert 1e13 < rate < 1e14                      # tens of T lane-ops/s on any gfx950 part
    assert B.load().alpa_dp_measure_valu_peak(None) == -1
    # the usage example of the README: solve, then place the chosen submeshes
    w = W.make_workload(2)
    h = B.alpa_dp_create(w.table, w.K, w.N, w.M, w.B, w.shapes)
    try:
        T, plan = B.alpa_dp_solve(h, None, 0, B.ALPA_DP_PRUNE)
        shapes = [tuple(int(x) for x in w.shapes[q]) for q in plan["shape_idx"]]
        where = B.alpa_place_submeshes(w.N, w.M, shapes)
        from oracle import placement
        assert where == placement.place(w.N, w.M, shapes)
        assert sum(n * m for n, m in shapes) == w.N * w.M
    finally:
        B.alpa_dp_destroy(h)


@pytest.mark.parametrize("case", [c for c in RANDOM_CASES if c[1] <= 64 and c[2] * c[3] <= 64],
                         ids=lambda c: f"s{c[0]}-K{c[1]}-{c[2]}x{c[3]}")
def test_random_tables_two_candidates_per_workgroup(case):
    """The register/LDS kernel takes two candidates per workgroup (and packs them into one
    pass where it can) only for long candidate lists; the tuning call forces that form
    here, on unstructured tables where most half-blocks need the entry-wise filter, odd
    candidate counts included."""
    seed, K, N, M = case
    w = W.random_problem(500 + seed, K, N, M, inf_frac=0.25, value_hi=[6, 80, 7000][seed % 3])
    cand_ref = oracle.all_candidates(w.table, w.shapes)
    if len(cand_ref) > 301:
        cand_ref = oracle.quantiles(cand_ref, 301)
    if len(cand_ref) == 0:
        pytest.skip("no finite entry")
    for prune in (False, True):
        T_ref, p_ref = oracle.solve_parallel(w.table, w.N, w.M, w.B, w.shapes, cand_ref, prune, 8)
        h = B.alpa_dp_create(w.table, w.K, w.N, w.M, w.B, w.shapes)
        try:
            B.alpa_dp_set_tuning(h, B.ALPA_DP_TUNE_CANDIDATES_PER_WG, 2)
            T, plan = B.alpa_dp_solve(h, cand_ref, flags=B.ALPA_DP_PRUNE if prune else 0)
            assert (T == T_ref).all()
            _same_plan(plan, p_ref)
        finally:
            B.alpa_dp_destroy(h)


def test_two_handles_on_two_streams_do_not_disturb_each_other():
    import torch
    wa, wb = W.make_workload(2), W.random_problem(41, 30, 4, 4, inf_frac=0.2, value_hi=300)
    ca = oracle.quantiles(oracle.all_candidates(wa.table, wa.shapes), 700)
    cb = oracle.quantiles(oracle.all_candidates(wb.table, wb.shapes), 500)
    Ta, pa = oracle.solve_parallel(wa.table, wa.N, wa.M, wa.B, wa.shapes, ca, False, 8)
    Tb, pb = oracle.solve_parallel(wb.table, wb.N, wb.M, wb.B, wb.shapes, cb, False, 8)
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    ha = B.alpa_dp_create(wa.table, wa.K, wa.N, wa.M, wa.B, wa.shapes)
    hb = B.alpa_dp_create(wb.table, wb.K, wb.N, wb.M, wb.B, wb.shapes)
    try:
        B.alpa_dp_set_stream(ha, sa)
        B.alpa_dp_set_stream(hb, sb)
        da = torch.from_numpy(ca.copy()).cuda(); db = torch.from_numpy(cb.copy()).cuda()
        oa = torch.empty(len(ca), dtype=torch.int64, device="cuda")
        ob = torch.empty(len(cb), dtype=torch.int64, device="cuda")
        qa = torch.zeros(B.PLAN_BYTES, dtype=torch.uint8, device="cuda")
        qb = torch.zeros(B.PLAN_BYTES, dtype=torch.uint8, device="cuda")
        torch.cuda.synchronize()
        for _ in range(5):                         # queued alternately, nothing waited for
            B.alpa_dp_solve_dev(ha, da, len(ca), 0, oa, qa)
            B.alpa_dp_solve_dev(hb, db, len(cb), 0, ob, qb)
        sa.synchronize(); sb.synchronize()
        assert (oa.cpu().numpy() == Ta).all() and (ob.cpu().numpy() == Tb).all()
        _same_plan(B.plan_from_bytes(qa.cpu().numpy().tobytes()), pa)
        _same_plan(B.plan_from_bytes(qb.cpu().numpy().tobytes()), pb)
    finally:
        B.alpa_dp_destroy(ha)
        B.alpa_dp_destroy(hb)


def test_create_and_destroy_give_the_memory_back():
    import torch
    w = W.make_workload(2)
    def cycle(n):
        for _ in range(n):
            h = B.alpa_dp_create(w.table, w.K, w.N, w.M, w.B, w.shapes)
            B.alpa_dp_solve_sweep(h, None, [2, 8])
            B.alpa_dp_destroy(h)
    cycle(3)
    torch.cuda.synchronize()
    free0, _ = torch.cuda.mem_get_info()
    cycle(40)
    torch.cuda.synchronize()
    free1, _ = torch.cuda.mem_get_info()
    assert free0 - free1 < 64 << 20                # no growth with the number of handles


WIDE_CASES = [  # seed, K, N, M: 65..128 devices, K <= 64: the two-window form of the fast kernel
    (60, 40, 10, 8), (61, 64, 16, 8), (62, 33, 9, 8), (63, 20, 3, 32), (64, 57, 2, 64),
    (65, 12, 33, 2), (66, 64, 13, 8), (67, 5, 4, 32),
]


@pytest.mark.parametrize("kernel", list(KERNELS))
@pytest.mark.parametrize("case", WIDE_CASES, ids=lambda c: f"s{c[0]}-K{c[1]}-{c[2]}x{c[3]}")
def test_meshes_of_65_to_128_devices(case, kernel):
    seed, K, N, M = case
    rng = np.random.default_rng(seed)
    w = W.random_problem(seed, K, N, M, inf_frac=float(rng.choice([0.0, 0.2, 0.5])),
                         value_hi=int(rng.choice([6, 60, 6000])))
    cand_ref = oracle.all_candidates(w.table, w.shapes)
    if len(cand_ref) > 150:
        cand_ref = oracle.quantiles(cand_ref, 150)
    for prune in (False, True):
        T_ref, p_ref = oracle.solve_parallel(w.table, w.N, w.M, w.B, w.shapes, cand_ref, prune, 8)
        h = B.alpa_dp_create(w.table, w.K, w.N, w.M, w.B, w.shapes)
        try:
            flags = KERNELS[kernel] | (B.ALPA_DP_PRUNE if prune else 0)
            T, plan = B.alpa_dp_solve(h, cand_ref, flags=flags)
            assert (T == T_ref).all()
            _same_plan(plan, p_ref)
            if not prune:
                plans = B.alpa_dp_solve_sweep(h, cand_ref, [1, w.B, 50], flags=flags)
                _same_plan(plans[1], p_ref)
        finally:
            B.alpa_dp_destroy(h)


DEEP_CASES = [  # seed, K, N, M: 65..128 layers (5-8 waves per workgroup), the last four on
    # 65..128 devices (two windows, stage counts up to 128)
    (70, 65, 4, 8), (71, 80, 8, 8), (72, 96, 2, 8), (73, 128, 8, 8), (74, 100, 1, 8),
    (75, 113, 4, 16), (76, 128, 3, 4), (77, 81, 1, 1),
    (78, 70, 9, 8), (79, 100, 16, 8), (80, 128, 2, 64), (81, 128, 16, 8),
]


@pytest.mark.parametrize("kernel", list(KERNELS))
@pytest.mark.parametrize("case", DEEP_CASES, ids=lambda c: f"s{c[0]}-K{c[1]}-{c[2]}x{c[3]}")
def test_models_of_65_to_128_layers(case, kernel):
    seed, K, N, M = case
    rng = np.random.default_rng(seed)
    w = W.random_problem(seed, K, N, M, inf_frac=float(rng.choice([0.0, 0.2, 0.5])),
                         value_hi=int(rng.choice([6, 60, 6000])))
    cand_ref = oracle.all_candidates(w.table, w.shapes)
    n_q = 60 if K * N * M <= 8192 else 20          # the oracle's time on the largest sizes
    if len(cand_ref) > n_q:
        cand_ref = oracle.quantiles(cand_ref, n_q)
    for prune in (False, True):
        T_ref, p_ref = oracle.solve_parallel(w.table, w.N, w.M, w.B, w.shapes, cand_ref, prune, 8)
        h = B.alpa_dp_create(w.table, w.K, w.N, w.M, w.B, w.shapes)
        try:
            flags = KERNELS[kernel] | (B.ALPA_DP_PRUNE if prune else 0)
            T, plan = B.alpa_dp_solve(h, cand_ref, flags=flags)
            assert (T == T_ref).all()
            _same_plan(plan, p_ref)
            if not prune:
                plans = B.alpa_dp_solve_sweep(h, cand_ref, [1, w.B, 50], flags=flags)
                _same_plan(plans[1], p_ref)
        finally:
            B.alpa_dp_destroy(h)


@pytest.mark.parametrize("kernel", list(KERNELS))
@pytest.mark.parametrize("case", [(1, 128, 16, 8, 65), (2, 100, 16, 8, 65), (3, 90, 9, 8, 40),
                                  (4, 64, 16, 8, 50), (5, 128, 8, 8, 50)],
                         ids=lambda c: f"s{c[0]}-K{c[1]}-{c[2]}x{c[3]}")
def test_plans_of_many_stages(case, kernel):
    """Optima with up to 100 stages (more than 64 on the 16x8 mesh): the upper stage counts of
    the recurrence, of the early-stop table and of plan recovery."""
    seed, K, N, M, at_least = case
    w = W.many_stage_problem(seed, K, N, M)
    cand_ref = oracle.quantiles(oracle.all_candidates(w.table, w.shapes), 16)
    T_ref, p_ref = oracle.solve_parallel(w.table, w.N, w.M, w.B, w.shapes, cand_ref, False, 8)
    assert p_ref.num_stages >= at_least
    h = B.alpa_dp_create(w.table, w.K, w.N, w.M, w.B, w.shapes)
    try:
        T, plan = B.alpa_dp_solve(h, cand_ref, flags=KERNELS[kernel])
        assert (T == T_ref).all()
        _same_plan(plan, p_ref)
    finally:
        B.alpa_dp_destroy(h)


@pytest.mark.parametrize("nc", [1, 2])
@pytest.mark.parametrize("case", [(1, 128, 8, 8), (2, 96, 4, 8), (3, 72, 2, 8)],
                         ids=lambda c: f"s{c[0]}-K{c[1]}-{c[2]}x{c[3]}")
def test_deep_formula_tables(case, nc):
    """Structured tables (monotone in the stage span, memory-bound infeasibility) are where
    the early stop of the column loops and the packed two-candidate passes take effect."""
    seed, K, N, M = case
    w = W.deep_model_problem(seed, K, N, M)
    cand_ref = oracle.quantiles(oracle.all_candidates(w.table, w.shapes), 121)
    for prune in (False, True):
        T_ref, p_ref = oracle.solve_parallel(w.table, w.N, w.M, w.B, w.shapes, cand_ref, prune, 8)
        assert (T_ref < oracle.INF64).any()
        h = B.alpa_dp_create(w.table, w.K, w.N, w.M, w.B, w.shapes)
        try:
            B.alpa_dp_set_tuning(h, B.ALPA_DP_TUNE_CANDIDATES_PER_WG, nc)
            T, plan = B.alpa_dp_solve(h, cand_ref, flags=B.ALPA_DP_PRUNE if prune else 0)
            assert (T == T_ref).all()
            _same_plan(plan, p_ref)
        finally:
            B.alpa_dp_destroy(h)


@pytest.mark.parametrize("force_sort", [False, True])
@pytest.mark.parametrize("case", [  # seed, K, N, M, largest value
    (90, 6, 2, 2, 50_000_000), (91, 9, 1, 4, (1 << 19) - 1), (92, 9, 1, 4, 1 << 19),
    (93, 40, 4, 4, 3000), (94, 1, 1, 1, 7), (95, 12, 2, 8, 1), (96, 33, 8, 8, 400_000),
], ids=lambda c: f"s{c[0]}-K{c[1]}-max{c[4]}")
def test_candidate_list_by_bitmap_and_by_sort(case, force_sort):
    """The ascending distinct finite table values (the candidates when no list is given) come
    from a presence bitmap when the largest value is below 2^19 and from a radix sort
    otherwise; both against the oracle's list, with zeros, the extreme values present, and the
    tuning call that forces the sort."""
    seed, K, N, M, hi = case
    w = W.random_problem(seed, K, N, M, inf_frac=0.3, value_hi=hi)
    tab = w.table.copy()
    fin = np.argwhere(tab != oracle.INF32)
    if len(fin) >= 2:                               # make sure both ends of the range occur
        tab[tuple(fin[0])] = 0
        tab[tuple(fin[-1])] = hi
    ref = oracle.all_candidates(tab, w.shapes)
    h = B.alpa_dp_create(tab, K, N, M, w.B, w.shapes)
    try:
        assert B.alpa_dp_count_candidates(h) == len(ref)
        if force_sort:
            B.alpa_dp_set_tuning(h, B.ALPA_DP_TUNE_DISTINCT_BY_SORT, 1)
        T, plan = B.alpa_dp_solve(h, None, 0, 0)
        assert (B.alpa_dp_candidates(h) == ref).all()
        T_ref, p_ref = oracle.solve_parallel(tab, N, M, w.B, w.shapes, ref[:200], False, 8)
        assert (T[:200] == T_ref).all()
        nq = 17
        if len(ref) > nq:
            B.alpa_dp_solve(h, None, nq, 0)
            assert (B.alpa_dp_candidates(h) == oracle.quantiles(ref, nq)).all()
    finally:
        B.alpa_dp_destroy(h)


def test_candidate_list_much_longer_than_the_table():
    """A caller's list far longer than the table has entries (the per-candidate arrays grow),
    with repeats and values between and beyond the table's; then the table's own list again."""
    w = W.random_problem(77, 6, 2, 4, inf_frac=0.2, value_hi=900, B=5)
    rng = np.random.default_rng(5)
    tmax = rng.integers(0, 1200, size=60_000).astype(np.int32)
    uniq = np.unique(tmax)
    T_u, p_ref = oracle.solve_parallel(w.table, w.N, w.M, w.B, w.shapes, uniq, False, 8)
    lookup = dict(zip(uniq.tolist(), T_u.tolist()))
    h = B.alpa_dp_create(w.table, w.K, w.N, w.M, w.B, w.shapes)
    try:
        for kernel in KERNELS.values():
            T, plan = B.alpa_dp_solve(h, tmax, flags=kernel)
            assert T.tolist() == [lookup[int(x)] for x in tmax]
            _same_plan(plan, p_ref)
        ref = oracle.all_candidates(w.table, w.shapes)
        T2, _ = B.alpa_dp_solve(h, None, 0, 0)
        assert (B.alpa_dp_candidates(h) == ref).all()
        T2_ref, _ = oracle.solve_parallel(w.table, w.N, w.M, w.B, w.shapes, ref, False, 8)
        assert (T2 == T2_ref).all()
    finally:
        B.alpa_dp_destroy(h)
