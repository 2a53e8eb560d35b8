"""Pins of the table-construction oracle (Sec. 5.2, Eq. 5, Alg. 1's intra-op loop nest) against
things other than itself: a hand-worked example, limits, invariants, and the benchmark
workloads' tables, which separate array code generates."""
import itertools

import numpy as np
import pytest

import oracle
from paper_2201_12023_amd import workloads as W
from tests.table_cases import INF32, load_example


def test_hand_worked_example():
    t_l, ms, ma, dev, exp = load_example()
    got = oracle.build_table(t_l, ms, ma, dev)
    assert (got == exp).all()


@pytest.mark.parametrize("idx", [1, 2, 3, 4, 5])
def test_single_option_profiles_reproduce_the_workload_tables(idx):
    w = W.make_workload(idx)
    p = W.single_option_profiles(w)
    assert (oracle.build_table(p.t_l, p.mem_stage, p.mem_act, p.mem_device) == w.table).all()


def _python_table(p):
    """The definition once more, entry by entry in pure Python (tiny sizes only)."""
    K, S, O = p.K, p.S, p.O
    out = np.full((K, K, K, S), INF32, np.int64)
    for s, k, i, q in itertools.product(range(1, K + 1), range(K), range(K), range(S)):
        if i < k:
            continue
        fits = [int(p.t_l[k, i, q, o]) for o in range(O)
                if int(p.mem_stage[k, i, q, o]) + s * int(p.mem_act[k, i, q, o]) <= p.mem_device]
        out[s - 1, k, i, q] = min(fits, default=INF32)
    return out


@pytest.mark.parametrize("seed", range(6))
def test_entry_by_entry_on_random_profiles(seed):
    p = W.random_profiles(seed, K=2 + seed, S=1 + seed % 3, O=1 + seed % 4)
    assert (oracle.build_table(p.t_l, p.mem_stage, p.mem_act, p.mem_device) == _python_table(p)).all()


@pytest.mark.parametrize("seed", range(4))
def test_limits_and_invariants(seed):
    p = W.random_profiles(10 + seed, K=7, S=3, O=5)
    K = p.K
    t = oracle.build_table(p.t_l, p.mem_stage, p.mem_act, p.mem_device)
    # more remaining stages never make a stage faster (the fitting set only shrinks)
    assert (t[1:].astype(np.int64) >= t[:-1].astype(np.int64)).all()
    # below the diagonal: nothing
    kk, ii = np.tril_indices(K, -1)
    assert (t[:, kk, ii, :] == INF32).all()
    # unlimited memory: the fastest option, for every s
    big = oracle.build_table(p.t_l, p.mem_stage, p.mem_act, 2**60)
    fastest = p.t_l.min(axis=3)
    up = np.triu(np.ones((K, K), bool))
    assert (big[:, up, :] == fastest[up, :][None]).all()
    # no memory at all: only options that need none
    none = oracle.build_table(p.t_l, p.mem_stage + 1, p.mem_act, 0)
    assert (none == INF32).all()
    # option order does not matter; a duplicated option changes nothing
    perm = np.random.default_rng(seed).permutation(p.O)
    t2 = oracle.build_table(p.t_l[..., perm], p.mem_stage[..., perm], p.mem_act[..., perm],
                            p.mem_device)
    assert (t2 == t).all()
    dup = lambda a: np.concatenate([a, a[..., :1]], axis=3)
    assert (oracle.build_table(dup(p.t_l), dup(p.mem_stage), dup(p.mem_act), p.mem_device) == t).all()
    # an extra option can only lower entries; a larger device can only lower entries
    more = oracle.build_table(p.t_l, p.mem_stage, p.mem_act, p.mem_device + 7)
    assert (more.astype(np.int64) <= t).all()
    # scaling all memory figures and the device by the same factor changes nothing
    assert (oracle.build_table(p.t_l, p.mem_stage * 1000, p.mem_act * 1000,
                               p.mem_device * 1000) == t).all()


def test_threshold_of_eq5_is_inclusive():
    t_l = np.full((1, 1, 1, 1), 9, np.int32)
    ms = np.full((1, 1, 1, 1), 6, np.int64)
    ma = np.full((1, 1, 1, 1), 4, np.int64)
    assert oracle.build_table(t_l, ms, ma, 10)[0, 0, 0, 0] == 9      # 6 + 1 * 4 == 10 fits
    assert oracle.build_table(t_l, ms, ma, 9)[0, 0, 0, 0] == INF32


def test_s_multiplies_the_activation_term_only():
    # K = 4 single-layer stages; the option fits exactly up to s = 3
    K = 4
    t_l = np.full((K, K, 1, 1), 5, np.int32)
    ms = np.full((K, K, 1, 1), 100, np.int64)
    ma = np.full((K, K, 1, 1), 7, np.int64)
    t = oracle.build_table(t_l, ms, ma, 100 + 3 * 7)
    up = np.triu(np.ones((K, K), bool))
    assert (t[:3][:, up, 0] == 5).all() and (t[3][up, 0] == INF32).all()
