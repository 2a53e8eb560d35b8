"""Reader of the hand-worked table-construction example (tests/golden/table_example.txt)."""
import os

import numpy as np

INF32 = 2**31 - 1
_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "table_example.txt")


def load_example():
    """Returns (t_l, mem_stage, mem_act, mem_device, expected_table)."""
    head, opts, exps = {}, [], []
    for line in open(_PATH):
        line = line.split("#")[0].split()
        if not line:
            continue
        val = [INF32 if x == "INF" else int(x) for x in line[1:]]
        if line[0] == "opt":
            opts.append(val)
        elif line[0] == "exp":
            exps.append(val)
        else:
            head[line[0]] = val[0]
    K, S, O = head["K"], head["S"], head["O"]
    t_l = np.full((K, K, S, O), INF32, np.int32)
    ms = np.zeros((K, K, S, O), np.int64)
    ma = np.zeros((K, K, S, O), np.int64)
    for k, i, q, o, t, a, b in opts:
        t_l[k, i, q, o], ms[k, i, q, o], ma[k, i, q, o] = t, a, b
    exp = np.full((K, K, K, S), INF32, np.int32)
    for k, i, q, *vals in exps:
        assert len(vals) == K
        exp[:, k, i, q] = vals
    return t_l, ms, ma, head["mem_device"], exp
