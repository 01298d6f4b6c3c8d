#!/usr/bin/env python3
"""Writes tests/golden/oracle_trace_n5_d97.txt: the oracle's coefficients over six steps on a small,
fully specified input (a 31-bit linear congruential sequence mapped to multiples of 1/64 in
[-4, 4), so that every fp32 input is exact and no random-number library is involved).

The file pins the oracle against silent changes of its own arithmetic (steps O1-O7: Eq. 7, the
sorted momentum of Eq. 11 with beta = 0.9, the normalisation of Eq. 12-13).  It is written by
this script, which calls nothing but oracle/; regenerate it only together with a justified change
of the oracle:  python tests/golden/make_oracle_trace.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import adacons_oracle as o  # noqa: E402

N, D, STEPS, BETA = 5, 97, 6, 0.9
OUT = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_trace_n5_d97.txt")


def inputs():
    """STEPS matrices N x D; x_{k+1} = (1103515245 x_k + 12345) mod 2^31, value = (x >> 22) / 64 - 4,
    plus a common ramp so that the rows correlate."""
    x = 20241103
    for _ in range(STEPS):
        G = np.empty((N, D), dtype=np.float32)
        for i in range(N):
            for k in range(D):
                x = (1103515245 * x + 12345) % (1 << 31)
                G[i, k] = np.float32((x >> 22) / 64.0 - 4.0 + (k % 7) * 0.5)
        yield G


def trace():
    st = o.OracleState(N, beta=BETA)
    rows = []
    for G in inputs():
        out, info = o.aggregate(G, st)
        rows.append(np.concatenate([info["raw"], info["smoothed"], info["gamma"], out[:3], st.m]))
    return np.array(rows)


if __name__ == "__main__":
    np.savetxt(OUT, trace(), fmt="%.17e",
               header="per step: raw a_i (5), smoothed (5), gamma (5), out[0:3], state m (5); N=5 d=97 beta=0.9")
    print("wrote", OUT)
