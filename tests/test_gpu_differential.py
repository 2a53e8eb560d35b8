"""Differential test on the GPU: the register/LDS recurrence kernel against the general one (which
the parity tests pin to the oracle at the same sizes) on a few hundred seeded random problems —
layer counts 1..128, every mesh of up to 128 devices, unstructured and formula tables, all three
ways of giving candidates, pruning on and off, one and two candidates per workgroup.  A mismatch
is then settled by the oracle: every tenth case is also checked against it directly."""
import numpy as np
import pytest

import oracle
from paper_2201_12023_amd import binding as B
from paper_2201_12023_amd import workloads as W

pytestmark = pytest.mark.gpu

MESHES = [(N, M) for M in (1, 2, 4, 8, 16, 32, 64) for N in range(1, 129)
          if N * M <= 128 and N - 1 + M.bit_length() <= 64]
KEYS = ("T_star", "t_max", "num_stages", "n_evaluated", "first_layer", "shape_idx")


def _problem(rng):
    while True:
        N, M = MESHES[rng.integers(len(MESHES))]
        K = int(rng.choice([rng.integers(1, 17), rng.integers(17, 65), rng.integers(65, 129)],
                           p=[0.3, 0.5, 0.2]))
        if K * K * K * (N + 7) <= 30_000_000:
            break
    kind, seed = int(rng.integers(4)), int(rng.integers(1 << 30))
    if kind == 0:
        return W.random_problem(seed, K, N, M, inf_frac=float(rng.choice([0.0, 0.1, 0.4, 0.8])),
                                value_hi=int(rng.choice([2, 9, 100, 5000, 300000])))
    if kind == 1:
        return W.deep_model_problem(seed % 1000, K, N, M, B=int(rng.integers(1, 200)))
    if kind == 2:
        return W.many_stage_problem(seed % 1000, K, N, M, B=int(rng.integers(1, 2000)))
    return W.random_problem(seed, K, N, M, inf_frac=0.05, value_hi=50, B=int(rng.integers(1, 64)))


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_tuned_kernel_against_general_kernel(seed):
    rng = np.random.default_rng(seed)
    for case in range(100):
        w = _problem(rng)
        h = B.alpa_dp_create(w.table, w.K, w.N, w.M, w.B, w.shapes)
        try:
            nd = B.alpa_dp_count_candidates(h)
            mode = int(rng.integers(3))
            prune = B.ALPA_DP_PRUNE if rng.integers(2) else 0
            if nd == 0 or mode == 0:
                args = (None, min(nd, 2000) if nd > 2000 else 0)
            elif mode == 1 and nd > 2:
                args = (None, int(rng.integers(2, min(nd, 700) + 1)))
            else:
                hi = int(w.table[w.table != W.INF_I32].max(initial=5)) + 3
                args = (rng.integers(0, hi, size=int(rng.integers(1, 400))).astype(np.int32),)
            B.alpa_dp_set_tuning(h, B.ALPA_DP_TUNE_CANDIDATES_PER_WG,
                                 2 if rng.integers(3) == 0 else 0)
            T1, p1 = B.alpa_dp_solve(h, *args, flags=prune)
            T2, p2 = B.alpa_dp_solve(h, *args, flags=prune | B.ALPA_DP_GENERIC)
            what = f"seed {seed} case {case}: {w.name} K={w.K} {w.N}x{w.M} B={w.B} mode {mode} prune {prune}"
            assert (T1 == T2).all(), what
            assert all(p1[k] == p2[k] for k in KEYS), what
            cand = B.alpa_dp_candidates(h)[:64]
            if case % 10 == 0 and w.K * w.D <= 2048 and len(cand):
                T_o, _ = oracle.eval_candidates(w.table, w.N, w.M, w.B, w.shapes, cand, threads=8)
                T3, _ = B.alpa_dp_solve(h, cand, flags=0)
                assert (T3 == T_o).all(), what
        finally:
            B.alpa_dp_destroy(h)
