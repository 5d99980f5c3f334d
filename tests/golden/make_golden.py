"""Writes tests/golden/c1_oracle_rows.txt: the fp64 oracle's outputs for a few rows of the tiny
workload C1 (batch 1, 1 head, n=128, d=16, fp32 inputs).  The paper prints no worked numeric
example for this path, so this fixture is not a pin of the oracle (tests/test_oracle_pins.py
holds those); it guards the oracle and the input recipe against silent change.
Calls only oracle/ and the input generator.   Usage: python tests/golden/make_golden.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
import workloads  # noqa: E402

ROWS = [0, 1, 2, 15, 16, 17, 31, 64, 100, 127]


def main():
    w = workloads.C1
    Q, K, V = workloads.make_inputs(w)
    O = oracle.forward(Q, K, V, w.lam, w.scale, rows=ROWS)[0, 0]
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c1_oracle_rows.txt")
    with open(path, "w") as f:
        f.write("# oracle.forward on workloads.C1 (seed %d), lambda=%g scale=%g; row then %d values\n"
                % (workloads.SEED0 + w.index, w.lam, w.scale, w.d))
        for r, o in zip(ROWS, O):
            f.write("%d %s\n" % (r, " ".join("%.17g" % x for x in o)))
    print("wrote", path)


if __name__ == "__main__":
    main()
