"""ctypes front end of the float64 CPU oracle (``adacons_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke()``
and by the ``cpu_baseline`` leg of ``bench.py``.  It never imports the GPU
package and the GPU package never imports it.

All the method's arithmetic lives in the C file; this module only compiles it
(gcc, -O2, OpenMP, no fast-math), marshals numpy arrays and keeps the
sorted-order EMA state of Eq. 11 between calls.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "adacons_oracle.c")
_LIB = os.path.join(_HERE, "liboracle_adacons.so")
# The mutation tests point this at a deliberately broken build to prove the pins notice.
_LIB_OVERRIDE = os.environ.get("ADACONS_ORACLE_LIB_OVERRIDE")

F32 = 0
BF16 = 1
FLAG_MOMENTUM = 1
FLAG_NORMALIZE = 2
FLAG_INDEX_EMA = 4      # with FLAG_MOMENTUM: index-coupled EMA of Eq. 10 instead of the sorted one of Eq. 11
FLAG_LAMBDA_EQ13 = 8    # with FLAG_NORMALIZE: lambda as Eq. 13 prints it (sum of a~, not of the weights)
FLAG_DEFAULT = FLAG_MOMENTUM | FLAG_NORMALIZE
NUM_ZERO_NORM = 1
NUM_NONFINITE = 2
NUM_UNIFORM_FALLBACK = 4

_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle into a shared object next to its source."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared",
               "-fno-fast-math", "-ffp-contract=off", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _bind(path: str):
    """Open a built oracle library and declare its signatures."""
    lib = ctypes.CDLL(path)
    dp = ctypes.POINTER(ctypes.c_double)
    lib.oracle_num_threads.restype = ctypes.c_int
    lib.oracle_gram.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_int, dp]
    lib.oracle_coefficients.argtypes = [dp, ctypes.c_int, ctypes.c_double, ctypes.c_uint, dp,
                                        ctypes.POINTER(ctypes.c_int64), dp, dp, dp,
                                        ctypes.POINTER(ctypes.c_uint)]
    lib.oracle_coefficients_from_stats.argtypes = [dp, dp, ctypes.c_int, ctypes.c_double, ctypes.c_uint, dp,
                                                   ctypes.POINTER(ctypes.c_int64), dp, dp, dp,
                                                   ctypes.POINTER(ctypes.c_uint)]
    lib.oracle_weighted_sum.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int64,
                                        ctypes.c_int, dp, dp]
    lib.oracle_weighted_sum_at.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int64,
                                           ctypes.c_int, dp, ctypes.POINTER(ctypes.c_int64),
                                           ctypes.c_int64, dp]
    return lib


def _load():
    global _lib
    if _lib is None:
        _lib = _bind(_LIB_OVERRIDE if _LIB_OVERRIDE else build())
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_num_threads(n: int) -> None:
    """OpenMP threads used from now on (the results do not depend on the count)."""
    lib = _load()
    lib.oracle_set_num_threads.argtypes = [ctypes.c_int]
    lib.oracle_set_num_threads.restype = None
    lib.oracle_set_num_threads(int(n))


def _dp(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _as_input(G) -> tuple[np.ndarray, int]:
    """Accept an (N, d) float32 array, or an (N, d) uint16/int16 array of bf16 bit patterns."""
    G = np.asarray(G)
    if G.ndim != 2:
        raise ValueError("G must be N x d")
    if G.dtype == np.float32:
        return np.ascontiguousarray(G), F32
    if G.dtype in (np.uint16, np.int16):
        return np.ascontiguousarray(G.view(np.uint16)), BF16
    raise TypeError(f"unsupported input dtype {G.dtype}: float32, or uint16 holding bf16 bits")


@dataclass
class OracleState:
    """Carried state of Eq. 11: the EMA of the order statistics, in sorted order."""
    N: int
    beta: float = 0.99
    flags: int = FLAG_DEFAULT
    m: np.ndarray = field(default=None)
    t: int = 0

    def __post_init__(self):
        if self.m is None:
            self.m = np.zeros(self.N, dtype=np.float64)


def gram(G) -> np.ndarray:
    """Step O1: K = G G^T in float64 (Eq. 7, third line)."""
    G, dt = _as_input(G)
    N, d = G.shape
    K = np.empty((N, N), dtype=np.float64)
    rc = _load().oracle_gram(G.ctypes.data, N, d, dt, _dp(K))
    if rc:
        raise RuntimeError(f"oracle_gram failed rc={rc}")
    return K


def coefficients(K: np.ndarray, state: OracleState) -> dict:
    """Steps O2-O7 (weights): K -> gamma; advances ``state`` by one call."""
    K = np.ascontiguousarray(K, dtype=np.float64)
    N = state.N
    if K.shape != (N, N):
        raise ValueError("K must be N x N")
    gamma = np.empty(N)
    raw = np.empty(N)
    smooth = np.empty(N)
    t = ctypes.c_int64(state.t)
    nf = ctypes.c_uint(0)
    rc = _load().oracle_coefficients(_dp(K), N, state.beta, state.flags, _dp(state.m),
                                     ctypes.byref(t), _dp(gamma), _dp(raw), _dp(smooth),
                                     ctypes.byref(nf))
    if rc:
        raise RuntimeError(f"oracle_coefficients failed rc={rc}")
    state.t = int(t.value)
    return {"gamma": gamma, "raw": raw, "smoothed": smooth, "numeric_flags": int(nf.value), "K": K}


def coefficients_from_stats(q, r, state: OracleState) -> dict:
    """Steps O3-O7 (weights) from q_i = ||g_i||^2 and r_i = <g_i, sum_j g_j>, the per-worker
    statistics of Algorithm 1; advances ``state`` by one call."""
    q = np.ascontiguousarray(q, dtype=np.float64)
    r = np.ascontiguousarray(r, dtype=np.float64)
    N = state.N
    if q.shape != (N,) or r.shape != (N,):
        raise ValueError("q and r must have N entries")
    gamma, raw, smooth = np.empty(N), np.empty(N), np.empty(N)
    t = ctypes.c_int64(state.t)
    nf = ctypes.c_uint(0)
    rc = _load().oracle_coefficients_from_stats(_dp(q), _dp(r), N, state.beta, state.flags, _dp(state.m),
                                                ctypes.byref(t), _dp(gamma), _dp(raw), _dp(smooth),
                                                ctypes.byref(nf))
    if rc:
        raise RuntimeError(f"oracle_coefficients_from_stats failed rc={rc}")
    state.t = int(t.value)
    return {"gamma": gamma, "raw": raw, "smoothed": smooth, "numeric_flags": int(nf.value)}


def worker_stats(g, gsum) -> tuple[float, float, float]:
    """One worker's statistics in Algorithm 1: (||g||^2, <g, gsum>, ||gsum||^2) in float64, i.e. the
    Gram matrix of the two vectors (gsum = the all-reduced sum of the gradients, as stored)."""
    K = gram(np.ascontiguousarray(np.stack([np.asarray(g), np.asarray(gsum)])))
    return float(K[0, 0]), float(K[0, 1]), float(K[1, 1])


def weighted_sum(G, gamma) -> np.ndarray:
    """Step O7 (combination): out = sum_i gamma_i g_i in float64 (Eq. 12)."""
    G, dt = _as_input(G)
    N, d = G.shape
    gamma = np.ascontiguousarray(gamma, dtype=np.float64)
    out = np.empty(d, dtype=np.float64)
    rc = _load().oracle_weighted_sum(G.ctypes.data, N, d, dt, _dp(gamma), _dp(out))
    if rc:
        raise RuntimeError(f"oracle_weighted_sum failed rc={rc}")
    return out


def weighted_sum_at(G, gamma, idx) -> np.ndarray:
    """Eq. 12 at the listed columns only."""
    G, dt = _as_input(G)
    N, d = G.shape
    gamma = np.ascontiguousarray(gamma, dtype=np.float64)
    idx = np.ascontiguousarray(idx, dtype=np.int64)
    out = np.empty(idx.shape[0], dtype=np.float64)
    rc = _load().oracle_weighted_sum_at(G.ctypes.data, N, d, dt, _dp(gamma),
                                        idx.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
                                        idx.shape[0], _dp(out))
    if rc:
        raise RuntimeError(f"oracle_weighted_sum_at failed rc={rc}")
    return out


def aggregate(G, state: OracleState, want_out: bool = True) -> tuple[np.ndarray | None, dict]:
    """One whole aggregation O1-O7; returns (out or None, info dict)."""
    info = coefficients(gram(G), state)
    out = weighted_sum(G, info["gamma"]) if want_out else None
    return out, info


def aggregate_layers(G, offsets, states: list, want_out: bool = True):
    """Layer-wise aggregation (Sec. 4 of the paper): steps O1-O7 applied independently to every
    contiguous column segment G[:, offsets[l]:offsets[l+1]], each with its own state.
    Returns (out or None, list of per-layer info dicts)."""
    G = np.asarray(G)
    offsets = np.asarray(offsets, dtype=np.int64)
    L = offsets.shape[0] - 1
    if len(states) != L:
        raise ValueError("one OracleState per layer")
    out = np.empty(G.shape[1], dtype=np.float64) if want_out else None
    infos = []
    for l in range(L):
        a, b = int(offsets[l]), int(offsets[l + 1])
        seg = np.ascontiguousarray(G[:, a:b])
        o_l, info = aggregate(seg, states[l], want_out=want_out)
        if want_out:
            out[a:b] = o_l
        infos.append(info)
    return out, infos
