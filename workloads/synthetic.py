"""Seeded synthetic gradient streams shaped like the paper's workloads.

The paper measures on MLPerf v4.0 training tasks (ResNet-50 / ImageNet,
RetinaNet, DLRM, BERT-Large; Sec. 4); neither the datasets nor trained weights
are available here, so these streams take only the *shapes* of those workloads
(flattened parameter counts, worker counts) and stand in for them.

This module holds none of the aggregation arithmetic: it only draws inputs.
It serves the GPU tests, the benchmark and the CPU oracle's tests alike; the
random numbers come from ``torch.Generator`` on whichever device is asked for
(bits differ between CPU and GPU generators, which is fine: each parity test
feeds the *same* tensor to both sides).

Every gradient is  g_i = scale_i * (signal + sigma * noise_i)  with a shared
signal ``s`` (the consensus direction) and i.i.d. N(0, 1) per-worker noise.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace
from typing import Iterator

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    N: int                 # workers
    d: int                 # flattened gradient length
    dtype: str             # "f32" | "bf16" (storage type of G)
    steps: int
    sigma: float           # noise standard deviation relative to unit signal
    kind: str              # recipe selector, see ``stream``
    seed: int = 0

    def scaled(self, d: int, steps: int | None = None) -> "Workload":
        """Same recipe at another length / step count (parity-test sizes)."""
        return replace(self, d=int(d), steps=self.steps if steps is None else int(steps))

    @property
    def elem_bytes(self) -> int:
        return 2 if self.dtype == "bf16" else 4

    @property
    def floor_bytes(self) -> int:
        """Algorithmic bytes of one aggregation: G read twice, fp32 out written once."""
        return 2 * self.N * self.d * self.elem_bytes + 4 * self.d


# The five configurations of the benchmark definition.
C1 = Workload("C1-tiny", 4, 1_048_576, "f32", 1, 0.5, "plain")
C2 = Workload("C2-resnet50", 8, 25_557_032, "f32", 20, 1.0, "scaled_correlated")
C3 = Workload("C3-bertlarge-bf16", 8, 335_141_888, "bf16", 1, 2.0, "block_scaled")
C4 = Workload("C4-many-workers", 64, 25_557_032, "f32", 10, 3.0, "plain")
C5 = Workload("C5-robustness", 16, 124_439_808, "f32", 100, 1.0, "outlier_shuffled")
CONFIGS = {"C1": C1, "C2": C2, "C3": C3, "C4": C4, "C5": C5}
# Beside them: the shape of the paper's stochastic linear-regression example (Eq. 14: d = 1000, up to 128
# workers) -- many workers with few parameters each, bound by launches.  Not one of the five configurations;
# bench.py takes it as --workload E14 so that the figures quoted for this regime have a command behind them.
E14 = Workload("E14-many-workers-short-gradients", 128, 1000, "f32", 25, 1.0, "plain")
EXTRA = {"E14": E14}


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def stream(w: Workload, device="cpu") -> Iterator[torch.Tensor]:
    """Yield ``w.steps`` gradient matrices G_t (N x d, row-major, contiguous).

    kinds
      plain              g_i = s_t + sigma n_{i,t}; s_t, n redrawn every step (C1, C4)
      scaled_correlated  g_i = (1 + 0.1 i)(s_t + sigma n_{i,t});
                         s_t = 0.9 s_{t-1} + sqrt(1 - 0.81) z_t  (unit variance, lag-1 corr 0.9) (C2)
      block_scaled       g_i = f_b (s + sigma n_i), f_b = 10^U(-3,0) per 4096-element block,
                         the same for every worker; rounded once to bf16 when dtype is bf16 (C3)
      outlier_shuffled   N-1 workers s_t + sigma n_{i,t}, one worker -5 s_t + sigma n; then the rows
                         are permuted by a per-step seeded shuffle (C5)
    The yielded tensor is reused between steps: consume it before advancing.
    """
    dev = torch.device(device)
    gen = _gen(dev, w.seed)
    N, d = w.N, w.d
    buf = torch.empty((N, d), dtype=torch.float32, device=dev)
    s = torch.empty(d, dtype=torch.float32, device=dev)
    z = torch.empty(d, dtype=torch.float32, device=dev) if w.kind == "scaled_correlated" else None
    # permutations come from a CPU generator so that the order does not depend on the device
    pgen = _gen("cpu", w.seed + 7919)

    for t in range(w.steps):
        if w.kind == "scaled_correlated" and t > 0:
            z.normal_(generator=gen)
            s.mul_(0.9).add_(z, alpha=math.sqrt(1.0 - 0.81))
        else:
            s.normal_(generator=gen)
        buf.normal_(generator=gen)
        if w.sigma != 1.0:
            buf.mul_(w.sigma)

        if w.kind == "outlier_shuffled":
            buf[: N - 1].add_(s)
            buf[N - 1].add_(s, alpha=-5.0)
            perm = torch.randperm(N, generator=pgen).to(dev)
            G = buf.index_select(0, perm)
        else:
            buf.add_(s)
            if w.kind == "scaled_correlated":
                scale = 1.0 + 0.1 * torch.arange(N, dtype=torch.float32, device=dev)
                buf.mul_(scale[:, None])
            elif w.kind == "block_scaled":
                nblk = (d + 4095) // 4096
                u = torch.rand(nblk, generator=gen, dtype=torch.float32, device=dev)
                f = torch.pow(10.0, -3.0 * u)
                buf.mul_(f.repeat_interleave(4096)[:d][None, :])
            G = buf

        if w.dtype == "bf16":
            G = G.to(torch.bfloat16)      # round-to-nearest-even, once
        yield G.contiguous()


def to_oracle_input(G: torch.Tensor):
    """Host copy of G in the form the oracle takes: float32, or uint16 bf16 bit patterns."""
    import numpy as np
    G = G.detach()
    if G.dtype == torch.bfloat16:
        return G.view(torch.int16).cpu().numpy().view(np.uint16)
    if G.dtype == torch.float32:
        return G.cpu().numpy()
    raise TypeError(G.dtype)


def resnet50_layer_sizes() -> list[int]:
    """Element counts of the 161 parameter tensors of a ResNet-50 v1 (conv weights, batch-norm
    scale and shift, the final fully connected layer), in definition order, computed from the
    architecture: stem 7x7x3x64, bottleneck stages of [3, 4, 6, 3] blocks with widths
    [64, 128, 256, 512] and expansion 4, 1000-way classifier.  They add up to 25,557,032, the
    flattened gradient length of the C2 / C4 workloads; used as the layer layout of the
    layer-wise benchmark."""
    sizes = [7 * 7 * 3 * 64, 64, 64]
    inplanes = 64
    for width, blocks in zip([64, 128, 256, 512], [3, 4, 6, 3]):
        for b in range(blocks):
            sizes += [inplanes * width, width, width]            # 1x1 reduce + bn
            sizes += [3 * 3 * width * width, width, width]        # 3x3 + bn
            sizes += [width * width * 4, width * 4, width * 4]    # 1x1 expand + bn
            if b == 0:
                sizes += [inplanes * width * 4, width * 4, width * 4]   # projection shortcut + bn
            inplanes = width * 4
    sizes += [2048 * 1000, 1000]
    return sizes
