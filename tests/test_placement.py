"""Placement of a plan's submeshes (Sec. 5.2, Appendix A): pins of the oracle, and the library's
host-side routine against the oracle (no device is needed for either)."""
import itertools

import numpy as np
import pytest

from oracle import placement
from paper_2201_12023_amd import binding as B
from paper_2201_12023_amd import workloads as W


def _check_valid(N, M, shapes, pos):
    grid = -np.ones((N, M), int)
    for p, ((n, m), (r, c)) in enumerate(zip(shapes, pos)):
        assert 0 <= r and r + n <= N and 0 <= c and c + m <= M
        assert (grid[r:r + n, c:c + m] == -1).all()          # rectangles do not overlap
        grid[r:r + n, c:c + m] = p
        if n == 1:
            assert c % m == 0                                 # aligned, as in Appendix A
        else:
            assert c == 0 and m == M
    assert (grid >= 0).all()                                  # and they cover the mesh
    return grid


def _multisets(N, M):
    """Every multiset of family shapes whose device counts add up to N * M (small meshes)."""
    fam = [tuple(int(x) for x in s) for s in W.submesh_shapes(N, M)]
    out = []

    def rec(start, left, cur):
        if left == 0:
            out.append(list(cur))
            return
        for j in range(start, len(fam)):
            a = fam[j][0] * fam[j][1]
            if a <= left:
                cur.append(fam[j]); rec(j, left - a, cur); cur.pop()
    rec(0, N * M, [])
    return out


@pytest.mark.parametrize("N,M", [(1, 1), (1, 4), (2, 2), (3, 2), (2, 4), (3, 4)])
def test_every_shape_multiset_of_small_meshes(N, M):
    rng = np.random.default_rng(N * 10 + M)
    sets = _multisets(N, M)
    assert sets
    for ms in sets:
        for _ in range(3):
            shapes = [ms[j] for j in rng.permutation(len(ms))]       # any pipeline order
            pos = placement.place(N, M, shapes)
            grid = _check_valid(N, M, shapes, pos)
            # larger first: along the row-major scan device counts never increase
            scan = []
            for p in grid.ravel():
                if p not in scan:
                    scan.append(int(p))
            sizes = [shapes[p][0] * shapes[p][1] for p in scan]
            assert sizes == sorted(sizes, reverse=True)
            # stages of one shape appear in pipeline order
            for shp in set(shapes):
                same = [p for p in scan if shapes[p] == shp]
                assert same == sorted(same)
            # the library's routine gives the same positions
            assert B.alpa_place_submeshes(N, M, shapes) == pos


def test_hand_example():
    # 3 x 4 mesh; pipeline order: (1,2) (2,4) (1,1) (1,1)
    # largest first: (2,4) takes rows 0-1; then (1,2) at row 2 cols 0-1; then the two (1,1)
    pos = placement.place(3, 4, [(1, 2), (2, 4), (1, 1), (1, 1)])
    assert pos == [(2, 0), (0, 0), (2, 2), (2, 3)]
    assert B.alpa_place_submeshes(3, 4, [(1, 2), (2, 4), (1, 1), (1, 1)]) == pos


@pytest.mark.parametrize("seed", range(20))
def test_random_large_meshes(seed):
    rng = np.random.default_rng(seed)
    N, M = int(rng.integers(1, 17)), int(2 ** rng.integers(0, 5))
    fam = [tuple(int(x) for x in s) for s in W.submesh_shapes(N, M)]
    shapes, left_rows = [], N
    # whole rows for some 2-D submeshes, the rest in powers of two
    while left_rows >= 2 and rng.random() < 0.5:
        n = int(rng.integers(2, left_rows + 1))
        shapes.append((n, M)); left_rows -= n
    left = left_rows * M
    while left > 0:
        m = int(2 ** rng.integers(0, int(np.log2(M)) + 1))
        if m <= left and (1, m) in fam:
            shapes.append((1, m)); left -= m
    shapes = [shapes[j] for j in rng.permutation(len(shapes))]
    if len(shapes) > 256:
        pytest.skip("more stages than a plan can hold")
    pos = placement.place(N, M, shapes)
    _check_valid(N, M, shapes, pos)
    assert B.alpa_place_submeshes(N, M, shapes) == pos


def test_argument_errors():
    L = B.load()
    arr = (B.alpa_shape_t * 2)(B.alpa_shape_t(1, 2), B.alpa_shape_t(1, 2))
    row = np.zeros(2, np.int32); col = np.zeros(2, np.int32)
    ok = lambda N, M, n=2, a=arr: L.alpa_place_submeshes(N, M, a, n, row.ctypes.data, col.ctypes.data)
    assert ok(1, 4) == 0
    assert ok(2, 4) == -1                       # 4 devices for an 8-device mesh
    assert ok(1, 3) == -1                       # M not a power of two
    assert ok(1, 4, 0) == -1
    assert L.alpa_place_submeshes(1, 4, None, 2, row.ctypes.data, col.ctypes.data) == -1
    bad = (B.alpa_shape_t * 2)(B.alpa_shape_t(2, 2), B.alpa_shape_t(1, 4))
    assert ok(2, 4, 2, bad) == -1               # (2, 2) on a 2 x 4 mesh is outside the family
    with pytest.raises(ValueError):
        placement.place(2, 4, [(1, 2), (1, 2)])
