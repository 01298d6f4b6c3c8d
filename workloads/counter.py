"""Counter-based synthetic gradients: every value is a pure function of (seed, step, worker, index).

The streams in ``synthetic.py`` draw from ``torch.Generator``, whose bits depend on the torch build
and on the device; a trace made with them can only be reproduced on the same software and hardware.
Here a value is computed from its coordinates alone, in integer arithmetic plus operations that IEEE
arithmetic defines exactly, so the same inputs -- bit for bit -- come out on any machine, in any
order, for any slice of the index range:

  three 64-bit words  w_j = mix64(key(seed, step, worker) + (3 index + j) * GOLDEN),  j = 0, 1, 2
  (mix64 = the SplitMix64 finaliser), cut into twelve 16-bit fields u_1 .. u_12;
  n = (u_1 + ... + u_12 - 6 * 65535) / 65536          (exact in fp32: the sum is below 2^24)

i.e. the classic twelve-uniform (Irwin-Hall) stand-in for a standard normal: mean 0, variance
1 - 2^-32, support +-6.  The recipes on top of it are those of the five benchmark configurations
(see ``synthetic.stream``), evaluated in numpy float32 one operation at a time (no fused
multiply-add), so they round identically everywhere.

This module holds none of the aggregation arithmetic; it only draws inputs (numpy, host side).
"""
from __future__ import annotations

import math
from typing import Iterator

import numpy as np

from .synthetic import Workload

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
# stream ids above any worker index
SIGNAL, INNOVATION, BLOCK_SCALE, SHUFFLE = 1 << 20, (1 << 20) + 1, (1 << 20) + 2, (1 << 20) + 3


def mix64(x: np.ndarray) -> np.ndarray:
    """SplitMix64 finaliser on an array of uint64 (arithmetic modulo 2^64)."""
    x = np.asarray(x, dtype=np.uint64).copy()
    x ^= x >> np.uint64(30)
    x *= _M1
    x ^= x >> np.uint64(27)
    x *= _M2
    x ^= x >> np.uint64(31)
    return x


def _key(seed: int, step: int, worker: int) -> np.uint64:
    k = mix64(np.array([seed], dtype=np.uint64) * _GOLDEN + np.uint64(1))
    k = mix64(k ^ (np.array([step], dtype=np.uint64) * _M1))
    k = mix64(k ^ (np.array([worker], dtype=np.uint64) * _M2))
    return k[0]


def words(seed: int, step: int, worker: int, start: int, n: int, per_index: int = 3) -> np.ndarray:
    """(n, per_index) uint64 words of the indices start .. start + n - 1."""
    idx = np.arange(start, start + n, dtype=np.uint64)[:, None] * np.uint64(per_index) + np.arange(per_index, dtype=np.uint64)[None, :]
    return mix64(_key(seed, step, worker) + idx * _GOLDEN)


def normal(seed: int, step: int, worker: int, n: int, start: int = 0) -> np.ndarray:
    """n float32 values, approximately N(0, 1), of the indices start .. start + n - 1."""
    w = words(seed, step, worker, start, n)
    total = np.zeros(n, dtype=np.int64)
    for j in range(3):
        for shift in (0, 16, 32, 48):
            total += ((w[:, j] >> np.uint64(shift)) & np.uint64(0xFFFF)).astype(np.int64)
    return ((total - 6 * 65535).astype(np.float32)) / np.float32(65536.0)


def uniform(seed: int, step: int, worker: int, n: int, start: int = 0) -> np.ndarray:
    """n float32 values in [0, 1) with 24 random bits each."""
    w = words(seed, step, worker, start, n, per_index=1)[:, 0]
    return (w >> np.uint64(40)).astype(np.float32) / np.float32(1 << 24)


def permutation(seed: int, step: int, N: int) -> np.ndarray:
    """A permutation of 0 .. N-1: the stable order of N hash words."""
    return np.argsort(words(seed, step, SHUFFLE, 0, N, per_index=1)[:, 0], kind="stable")


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round to nearest even (finite inputs)."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    return ((b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)).astype(np.uint16)


def stream(w: Workload) -> Iterator[np.ndarray]:
    """The recipe of workload ``w`` (same kinds as ``synthetic.stream``) from the counter-based
    generator: yields ``w.steps`` host arrays, float32 (N, d), or uint16 bf16 bit patterns when
    ``w.dtype`` is "bf16".  A fresh array every step."""
    N, d, seed = w.N, w.d, w.seed
    f32 = np.float32
    s = None
    for t in range(w.steps):
        if w.kind == "scaled_correlated" and t > 0:
            z = normal(seed, t, INNOVATION, d)
            s = s * f32(0.9) + z * f32(math.sqrt(1.0 - 0.81))
        else:
            s = normal(seed, t, SIGNAL, d)
        G = np.empty((N, d), dtype=np.float32)
        for i in range(N):
            G[i] = normal(seed, t, i, d)
        if w.sigma != 1.0:
            G *= f32(w.sigma)
        if w.kind == "outlier_shuffled":
            G[: N - 1] += s[None, :]
            G[N - 1] += s * f32(-5.0)
            G = np.ascontiguousarray(G[permutation(seed, t, N)])
        else:
            G += s[None, :]
            if w.kind == "scaled_correlated":
                G *= (f32(1.0) + f32(0.1) * np.arange(N, dtype=np.float32))[:, None]
            elif w.kind == "block_scaled":
                nblk = (d + 4095) // 4096
                # 10^(-3 u) in float64, rounded once to float32: the only step here that leans on libm (pow is
                # not correctly rounded everywhere); two libms agree on the float32 result unless the float64
                # value sits within an ulp of a float32 rounding boundary, about 2^-29 per factor
                u = uniform(seed, t, BLOCK_SCALE, nblk).astype(np.float64)
                f = np.power(10.0, -3.0 * u).astype(np.float32)
                G *= np.repeat(f, 4096)[:d][None, :]
        yield to_bf16_bits(G) if w.dtype == "bf16" else G
