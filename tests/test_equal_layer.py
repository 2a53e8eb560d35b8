"""The "Equal layer" variant of the inter-op ablation study (Sec. 8.3): oracle pins on the CPU,
then the library's restricted handle against the oracle on the GPU."""
import numpy as np
import pytest

import oracle
from paper_2201_12023_amd import binding as B
from paper_2201_12023_amd import workloads as W
from tests import bruteforce as bf

INF32 = 2**31 - 1


@pytest.mark.parametrize("seed", range(12))
def test_masked_table_solves_to_the_best_equal_slicing(seed):
    """Enumeration of every plan (Eq. 2) restricted to plans whose stages have one length,
    against the recurrence on the masked table."""
    rng = np.random.default_rng(seed)
    K = int(rng.choice([1, 2, 3, 4, 6]))
    N, M = [(1, 2), (2, 2), (1, 4), (2, 1)][seed % 4]
    w = W.random_problem(300 + seed, K, N, M, inf_frac=0.1, value_hi=30)
    sizes = [int(x) for x in w.sizes]
    plans = [(st, lat) for st, lat in bf.enumerate_plans(w.table, K, w.D, sizes)
             if len({i - k + 1 for k, i, _ in st}) == 1]
    masked = oracle.equal_layer_table(w.table)
    cand = oracle.all_candidates(masked, w.shapes)
    if len(cand) == 0:
        assert not plans
        return
    T, plan = oracle.solve(masked, N, M, w.B, w.shapes, cand, False)
    if not plans:
        assert plan.T_star == oracle.INF64
        return
    best = min(sum(lat) + (w.B - 1) * max(lat) for _, lat in plans)
    assert plan.T_star == best
    lens = {b - a for a, b in zip(plan.first_layer[:-1], plan.first_layer[1:])}
    assert len(lens) == 1


def test_mask_keeps_exactly_the_equal_length_entries():
    K = 6
    t = np.zeros((K, K, K, 1), np.int32)
    m = oracle.equal_layer_table(t)
    kept = {(s + 1, k, i) for s, k, i in zip(*np.nonzero(m[..., 0] == 0))}
    want = {(s, k, k + (K - k) // s - 1) for s in range(1, K + 1) for k in range(K)
            if (K - k) % s == 0}
    assert kept == want
    # e.g. 6 layers in 3 stages: (3, 0, 1), then (2, 2, 3), then (1, 4, 5)
    assert {(3, 0, 1), (2, 2, 3), (1, 4, 5)} <= kept and (2, 0, 1) not in kept


@pytest.mark.gpu
@pytest.mark.parametrize("idx", [1, 2, 5, "deep"])
def test_restricted_handle_against_the_oracle(idx):
    # "deep": 96 layers on a 2x8 mesh, the 6-wave form of the register/LDS kernel
    w = W.deep_model_problem(5, 96, 2, 8) if idx == "deep" else W.make_workload(idx)
    masked = oracle.equal_layer_table(w.table)
    cand = oracle.all_candidates(masked, w.shapes)
    cand_q = oracle.quantiles(cand, 40)
    T_ref, p_ref = oracle.solve_parallel(masked, w.N, w.M, w.B, w.shapes, cand_q, False, 8)
    _, p_full = oracle.solve_parallel(w.table, w.N, w.M, w.B, w.shapes, cand_q, False, 8)
    assert p_ref.T_star >= p_full.T_star           # a restriction never helps
    h = B.alpa_dp_create(w.table, w.K, w.N, w.M, w.B, w.shapes)
    try:
        B.alpa_dp_solve(h, None, 0, 0)             # something to reset
        B.alpa_dp_restrict_equal_layers(h)
        assert (B.alpa_dp_get_table(h, w.K, w.S) == masked).all()
        assert B.alpa_dp_count_candidates(h) == len(cand)
        for flags in (0, B.ALPA_DP_GENERIC):
            T, plan = B.alpa_dp_solve(h, None, 40, flags)
            assert (B.alpa_dp_candidates(h) == cand_q).all()
            assert (T == T_ref).all()
            for key in ("T_star", "t_max", "num_stages", "first_layer", "shape_idx"):
                assert plan[key] == getattr(p_ref, key), key
        best = B.alpa_dp_best(h)
        assert best["T_star"] == p_ref.T_star
    finally:
        B.alpa_dp_destroy(h)


@pytest.mark.gpu
def test_restricting_twice_changes_nothing_and_null_is_rejected():
    w = W.random_problem(9, 12, 2, 4, inf_frac=0.2, value_hi=50)
    masked = oracle.equal_layer_table(w.table)
    h = B.alpa_dp_create(w.table, w.K, w.N, w.M, w.B, w.shapes)
    try:
        B.alpa_dp_restrict_equal_layers(h)
        B.alpa_dp_restrict_equal_layers(h)
        assert (B.alpa_dp_get_table(h, w.K, w.S) == masked).all()
        assert B.load().alpa_dp_restrict_equal_layers(None) == -1
    finally:
        B.alpa_dp_destroy(h)
