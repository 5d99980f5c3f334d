import os

import numpy as np

import oracle
import workloads


def test_c1_oracle_rows_fixture():
    path = os.path.join(os.path.dirname(__file__), "golden", "c1_oracle_rows.txt")
    rows, vals = [], []
    for line in open(path):
        if line.startswith("#"):
            continue
        parts = line.split()
        rows.append(int(parts[0]))
        vals.append([float(x) for x in parts[1:]])
    w = workloads.C1
    Q, K, V = workloads.make_inputs(w)
    O = oracle.forward(Q, K, V, w.lam, w.scale, rows=rows)[0, 0]
    assert np.abs(O - np.asarray(vals)).max() <= 1e-9
