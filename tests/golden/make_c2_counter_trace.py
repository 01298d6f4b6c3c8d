#!/usr/bin/env python3
"""Writes tests/golden/c2_counter_trace_n8_d262184.txt: the weights gamma of all 20 steps of the
C2 recipe (N = 8, scale heterogeneity 1 + 0.1 i, signal correlated 0.9 from step to step, beta = 0.99)
at the reduced length d = 262,184, with inputs from the counter-based generator (workloads/counter.py:
every value a pure function of seed, step, worker and index, reproducible bit for bit on any machine).

Calls nothing but the oracle and the input generator.  The file is what any box -- CPU oracle or GPU
library fed the same generated inputs -- must reproduce; it is a stored trace of the oracle, not an
independent pin of it.
"""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import workloads  # noqa: E402
from oracle import adacons_oracle as o  # noqa: E402

D = 262_184
OUT = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c2_counter_trace_n8_d262184.txt")


def trace():
    w = workloads.C2.scaled(D, 20)
    st = o.OracleState(w.N, beta=0.99)
    rows = []
    for G in workloads.counter.stream(w):
        _, info = o.aggregate(G, st, want_out=False)
        rows.append(info["gamma"].copy())
    return rows


if __name__ == "__main__":
    with open(OUT, "w") as fh:
        fh.write("# gamma per step (20 steps x 8 workers), C2 recipe at d=262184, counter-based inputs seed 0, beta 0.99;\n")
        fh.write("# written by tests/golden/make_c2_counter_trace.py from oracle/ only\n")
        for g in trace():
            fh.write(" ".join("%.17g" % v for v in g) + "\n")
    print("wrote", OUT)
