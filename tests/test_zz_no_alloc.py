"""The allocation-free variant of the operator-clustering entry point against the ordinary one:
``alpa_cluster_layers_static`` (device pointers, kernels only, work memory in a fixed array of
the library's device image) must return what ``alpa_cluster_layers`` returns, on two calls in a
row of which the second is smaller (the work array keeps the first call's contents), must not
change the amount of free device memory, and must report bad device-resident inputs through its
status word instead of faulting."""
import ctypes

import numpy as np
import pytest

from paper_2201_12023_amd import binding as B
from paper_2201_12023_amd import workloads as W

pytestmark = pytest.mark.gpu

INF64 = B.INF_I64


def _static(g, L, delta_ppm, stream=None):
    import torch
    with torch.cuda.stream(stream) if stream is not None else torch.cuda.stream(torch.cuda.current_stream()):
        d_flop = torch.from_numpy(np.ascontiguousarray(g.flop, np.int32)).cuda()
        d_src = torch.from_numpy(np.ascontiguousarray(g.src, np.int32)).cuda()
        d_dst = torch.from_numpy(np.ascontiguousarray(g.dst, np.int32)).cuda()
        d_nb = torch.from_numpy(np.ascontiguousarray(g.nbytes, np.int64)).cuda()
        d_out = torch.full((3,), 77, dtype=torch.int64, device="cuda")
        d_first = torch.full((L + 1,), 77, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    free0, _ = torch.cuda.mem_get_info()
    B.alpa_cluster_layers_static(d_flop, d_src, d_dst, d_nb, L, delta_ppm, d_out, d_first, stream)
    torch.cuda.synchronize()
    free1, _ = torch.cuda.mem_get_info()
    out = d_out.cpu().numpy()
    return (int(out[0]), int(out[1]), int(out[2]), [int(x) for x in d_first.cpu().numpy()],
            free0 - free1)


def _same(g, L, delta_ppm, stream=None):
    ref = B.alpa_cluster_layers(g.flop, g.src, g.dst, g.nbytes, L, delta_ppm)
    comm, sumsq, status, first, grown = _static(g, L, delta_ppm, stream)
    assert status == 0
    assert comm == ref["comm"] and sumsq == ref["sumsq"]
    assert first == (ref["first_op"] if ref["first_op"] else [-1] * (L + 1))
    return grown


def test_static_work_memory_variant_equals_the_allocating_one():
    import torch
    big = W.make_op_graph(5, 40)                    # 482 operators, near the limit of 512
    assert 400 < big.K <= B.CLUSTER_STATIC_MAX_OPS
    small = W.make_op_graph(6, 7)
    _same(big, 48, 500000)                          # first call on the device: set-up included
    grown = _same(small, 9, 500000)                 # smaller, over the first call's leftovers
    assert grown == 0                               # no device memory was taken
    assert _same(big, 48, 500000) == 0
    # no clustering satisfies a zero tolerance on these graphs: INF, 0, first_op = -1
    _same(small, 9, 0)
    # unstructured graphs (zero-FLOP operators, parallel edges), on a stream of the caller's
    st = torch.cuda.Stream()
    for seed in range(6):
        g = W.random_op_graph(seed, 30 + 37 * seed, 4 * (30 + 37 * seed))
        _same(g, 1 + (7 * seed) % 12, [0, 200000, 10**9][seed % 3], st)
    one = W.random_op_graph(9, 1, 0)                # a single operator, no edges
    _same(one, 1, 0)


def test_static_variant_reports_bad_inputs_without_touching_memory_out_of_bounds():
    import torch
    g = W.make_op_graph(1, 3)
    L_ = B.load()
    ref = B.alpa_cluster_layers(g.flop, g.src, g.dst, g.nbytes, 4, 500000)

    class G:
        pass

    def variant(**kw):
        v = G()
        v.flop, v.src, v.dst, v.nbytes = (np.array(x, copy=True) for x in (g.flop, g.src, g.dst, g.nbytes))
        for k, (pos, val) in kw.items():
            getattr(v, k)[pos] = val
        return v

    for bad, code in ((variant(flop=(2, -1)), -1), (variant(src=(0, 10**6)), -1),
                      (variant(dst=(1, g.K)), -1), (variant(src=(2, -3)), -1),
                      (variant(nbytes=(1, -5)), -1), (variant(nbytes=(0, 2**62)), -2),
                      (variant(flop=(0, 2**31 - 1)), -2)):
        comm, sumsq, status, first, _ = _static(bad, 4, 500000)
        assert status == code and comm == INF64 and sumsq == 0 and first == [-1] * 5
    # and a good call right after them is unaffected
    comm, sumsq, status, first, _ = _static(g, 4, 500000)
    assert (status, comm, sumsq, first) == (0, ref["comm"], ref["sumsq"], ref["first_op"])
    # sizes beyond the fixed work memory are refused on the host, nothing is queued
    d = torch.zeros(8, dtype=torch.int64, device="cuda")
    i32 = torch.zeros(B.CLUSTER_STATIC_MAX_OPS + 2, dtype=torch.int32, device="cuda")
    p = lambda t: ctypes.c_void_p(int(t.data_ptr()))
    assert L_.alpa_cluster_layers_static(p(i32), B.CLUSTER_STATIC_MAX_OPS + 1, None, None, None, 0,
                                         2, 0, p(d), p(i32), None) == -1
    assert b"ALPA_CLUSTER_STATIC_MAX_OPS" in L_.alpa_dp_last_error()
    assert L_.alpa_cluster_layers_static(p(i32), 4, None, None, None, 0,
                                         B.CLUSTER_STATIC_MAX_OPS + 1, 0, p(d), p(i32), None) == -1
    assert L_.alpa_cluster_layers_static(None, 4, None, None, None, 0, 2, 0, p(d), p(i32), None) == -1
    assert L_.alpa_cluster_layers_static(p(i32), 4, None, None, None, 3, 2, 0, p(d), p(i32), None) == -1
