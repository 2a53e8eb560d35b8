"""Writes tests/golden/workload_<n>.json from the CPU oracle alone.

For each of the five seeded workloads: the candidate list the method derives from the table
(all distinct finite values, or 4096 quantiles), T*(t_max) of Eq. 4 for every candidate and
the plan Alg. 1 ends with, as computed by ``oracle/`` (thread-per-candidate driver for the
large ones).  Stored: counts, SHA-256 of the int32 candidate array and of the int64 T array
(little endian), every 97th T value, and the plan.  Nothing here touches the HIP library.

With ``--sweep`` it writes tests/golden/sweep_<n>.json instead: the plan Alg. 1 ends with for
each of several numbers of microbatches B (Sec. 5.2: B is found by enumeration), every one a
separate run of the oracle.

Run from the repository root:  python tests/golden/make_golden.py [--sweep] [workload numbers]
"""
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

import oracle  # noqa: E402
from paper_2201_12023_amd import workloads as W  # noqa: E402


def main(which):
    threads = int(os.environ.get("ORACLE_THREADS", "8"))
    for idx in which:
        w = W.make_workload(idx)
        t0 = time.time()
        cand = oracle.all_candidates(w.table, w.shapes)
        n_distinct = int(cand.size)
        if w.candidates == "quantiles":
            cand = oracle.quantiles(cand, w.n_quantiles)
        T, plan = oracle.solve_parallel(w.table, w.N, w.M, w.B, w.shapes, cand, w.prune, threads)
        out = dict(workload=idx, name=w.name, K=w.K, N=w.N, M=w.M, B=w.B, S=w.S,
                   prune=bool(w.prune), n_distinct=n_distinct, n_candidates=int(cand.size),
                   table_sha256=hashlib.sha256(w.table.tobytes()).hexdigest(),
                   cand_sha256=hashlib.sha256(cand.astype("<i4").tobytes()).hexdigest(),
                   T_sha256=hashlib.sha256(T.astype("<i8").tobytes()).hexdigest(),
                   T_every_97=[int(x) for x in T[::97]],
                   plan=dict(T_star=plan.T_star, t_max=plan.t_max, num_stages=plan.num_stages,
                             n_evaluated=plan.n_evaluated, first_layer=plan.first_layer,
                             shape_idx=plan.shape_idx),
                   layer_cost=[int(x) for x in w.layer_cost],
                   layer_mem=[int(x) for x in w.layer_mem],
                   layer_act=[int(x) for x in w.layer_act],
                   oracle_seconds=round(time.time() - t0, 2), oracle_threads=threads)
        path = os.path.join(ROOT, "tests", "golden", f"workload_{idx}.json")
        with open(path, "w") as f:
            json.dump(out, f, indent=1)
            f.write("\n")
        print(f"workload {idx}: {cand.size} candidates, T*={plan.T_star}, "
              f"{out['oracle_seconds']} s", flush=True)


SWEEP_B = [1, 8, 32, 128, 512]


def main_sweep(which):
    threads = int(os.environ.get("ORACLE_THREADS", "8"))
    for idx in which:
        w = W.make_workload(idx)
        t0 = time.time()
        cand = oracle.all_candidates(w.table, w.shapes)
        if w.candidates == "quantiles":
            cand = oracle.quantiles(cand, w.n_quantiles)
        plans = []
        for Bv in SWEEP_B:
            _, plan = oracle.solve_parallel(w.table, w.N, w.M, Bv, w.shapes, cand, w.prune, threads)
            plans.append(dict(B=Bv, T_star=plan.T_star, t_max=plan.t_max,
                              num_stages=plan.num_stages, n_evaluated=plan.n_evaluated,
                              first_layer=plan.first_layer, shape_idx=plan.shape_idx))
            print(f"workload {idx} B={Bv}: T*={plan.T_star} t_max={plan.t_max} "
                  f"stages={plan.num_stages}", flush=True)
        out = dict(workload=idx, prune=bool(w.prune), n_candidates=int(cand.size),
                   table_sha256=hashlib.sha256(w.table.tobytes()).hexdigest(), plans=plans,
                   oracle_seconds=round(time.time() - t0, 2), oracle_threads=threads)
        path = os.path.join(ROOT, "tests", "golden", f"sweep_{idx}.json")
        with open(path, "w") as f:
            json.dump(out, f, indent=1)
            f.write("\n")


if __name__ == "__main__":
    args = sys.argv[1:]
    if "--sweep" in args:
        main_sweep([int(a) for a in args if a != "--sweep"] or [3, 4, 5])
    else:
        main([int(a) for a in args] or [1, 2, 3, 4, 5])
