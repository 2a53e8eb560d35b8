"""CPU-side checks of the C ABI: the library loads, exports every symbol the header
declares, and rejects bad arguments before touching a device."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2201_12023_amd import binding as B
from paper_2201_12023_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "alpa_dp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(alpa_(?:dp|cluster|place)_[a-z_A-Z]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = B.load()
    names = _declared_symbols()
    assert set(names) == set(B.SYMBOLS)
    for n in names:
        assert hasattr(L, n), n


def test_plan_struct_size_matches_header():
    # int64 + 3 * int32 + (MAX_K + 1) * int32 + MAX_K * int32
    assert B.PLAN_BYTES == 8 + 12 + 4 * 257 + 4 * 256


def _create_rc(table, K, N, M, Bm, shapes):
    L = B.load()
    shp = np.ascontiguousarray(shapes, dtype=np.int32).reshape(-1, 2)
    arr = (B.alpa_shape_t * shp.shape[0])(*[B.alpa_shape_t(int(n), int(m)) for n, m in shp])
    h = ctypes.c_void_p()
    rc = L.alpa_dp_create(ctypes.byref(h), table.ctypes.data if table is not None else None,
                          K, N, M, Bm, arr, shp.shape[0])
    assert h.value is None or rc == 0
    return rc, L.alpa_dp_last_error().decode()


def test_create_rejects_bad_arguments_on_the_host():
    w = W.make_workload(1)
    t = w.table
    assert _create_rc(None, w.K, w.N, w.M, w.B, w.shapes)[0] == -1
    assert _create_rc(t, 0, w.N, w.M, w.B, w.shapes)[0] == -1
    assert _create_rc(t, 257, w.N, w.M, w.B, w.shapes)[0] == -1
    assert _create_rc(t, w.K, w.N, 3, w.B, w.shapes)[0] == -1            # M not a power of two
    assert _create_rc(t, w.K, w.N, w.M, 0, w.shapes)[0] == -1            # B < 1
    assert _create_rc(t, w.K, 64, 32, w.B, w.shapes)[0] == -1            # too many devices
    bad = w.shapes.copy(); bad[1] = (2, 2)                               # (n > 1, m < M)
    rc, msg = _create_rc(t, w.K, w.N, w.M, w.B, bad)
    assert rc == -1 and "family" in msg
    bad = w.shapes.copy(); bad[1] = (1, 3)
    assert _create_rc(t, w.K, w.N, w.M, w.B, bad)[0] == -1
    bad = w.shapes.copy(); bad[2] = (1, 8)                               # larger than the mesh
    assert _create_rc(t, w.K, w.N, w.M, w.B, bad)[0] == -1
    # (the range of the table's values is checked by a reduction on the device: GPU tests)


def test_null_handle_is_rejected():
    L = B.load()
    assert L.alpa_dp_solve(None, None, 0, 0, None, None) == -1
    assert L.alpa_dp_solve_dev(None, None, 0, 0, None, None) == -1
    Bs = np.asarray([1, 2], np.int32)
    out = (B.alpa_plan_t * 2)()
    assert L.alpa_dp_solve_sweep(None, None, 0, 0, Bs.ctypes.data, 2, ctypes.addressof(out)) == -1
    assert L.alpa_dp_best(None, None) == -1
    assert L.alpa_dp_set_B(None, 3) == -1
    L.alpa_dp_destroy(None)


def test_clustering_rejects_bad_arguments_on_the_host():
    flop = np.asarray([3, 1, 2, 2], np.int32)
    src = np.asarray([0, 1, 2], np.int32)
    dst = np.asarray([1, 2, 3], np.int32)
    nb = np.asarray([5, 5, 5], np.int64)

    def rc(flop=flop, src=src, dst=dst, nb=nb, E=3, K=4, L=2, delta=500000):
        L_ = B.load()
        out = (ctypes.c_int64(), ctypes.c_int64(), (ctypes.c_int32 * (max(L, 0) + 1))())
        return L_.alpa_cluster_layers(flop.ctypes.data if flop is not None else None, K,
                                      src.ctypes.data, dst.ctypes.data, nb.ctypes.data, E, L, delta,
                                      ctypes.byref(out[0]), ctypes.byref(out[1]), out[2], None)

    assert rc(flop=None) == -1
    assert rc(K=0) == -1 and rc(K=B.CLUSTER_MAX_OPS + 1) == -1
    assert rc(L=0) == -1 and rc(delta=-1) == -1 and rc(E=-1) == -1
    assert rc(flop=np.asarray([3, -1, 2, 2], np.int32)) == -1
    assert rc(src=np.asarray([0, 2, 2], np.int32)) == -1            # src >= dst
    assert rc(dst=np.asarray([1, 2, 4], np.int32)) == -1            # dst >= K
    assert rc(nb=np.asarray([5, -5, 5], np.int64)) == -1
    assert rc(flop=np.asarray([2**30, 2**30, 0, 0], np.int32)) == -2
    assert rc(nb=np.asarray([2**61, 2**61, 5], np.int64)) == -2
