#!/usr/bin/env python3
"""Stochastic linear regression of Sec. 5.1 (Eq. 14) driven through the aggregation library.

    min_w  f(w) = E_{zeta ~ U[0,1]^d} [ (w^T zeta)^2 / 2 ],   d = 1000,
    f(w) = w^T H w / 2  with  H = E[zeta zeta^T] = I / 12 + 1 1^T / 4.

Every step each of the N workers draws B samples and forms its mini-batch gradient
g_i = (1/B) sum_b zeta_b (zeta_b^T w); the N gradients are aggregated on the GPU either by the
plain mean or by adacons_aggregate, and w moves along the aggregated direction psi with the
step that is optimal for the true objective, eta = psi^T H w / psi^T H psi (the paper gives every
method its analytically optimal step; which expression it used is not stated, so this exact line
search on f is this demo's reading).  A functional demo of the small-d, launch-bound regime --
not a reproduction of the paper's figure.

    python examples/linear_regression.py --workers 32 --batch 64 --steps 200
"""
from __future__ import annotations

import argparse
import os
import sys

import torch

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


def true_loss(w: torch.Tensor) -> float:
    """f(w) = w^T H w / 2 with H = I/12 + 11^T/4, in fp64."""
    w = w.double()
    return float(0.5 * (w.dot(w) / 12.0 + 0.25 * w.sum() ** 2))


def hessian_times(v: torch.Tensor) -> torch.Tensor:
    return v / 12.0 + 0.25 * v.sum()


def worker_gradients(w: torch.Tensor, N: int, B: int, gen: torch.Generator) -> torch.Tensor:
    """N mini-batch gradients of (w^T zeta)^2 / 2, one row each (fp32, on w's device)."""
    zeta = torch.rand(N, B, w.numel(), generator=gen, device=w.device)
    r = zeta @ w                                 # [N, B] residuals w^T zeta
    return torch.einsum("nb,nbd->nd", r, zeta) / B


def run(aggregate, N: int, B: int, steps: int, d: int = 1000, seed: int = 0, device: str = "cuda:0"):
    """aggregate(G) -> psi (d floats on the device).  Returns the loss after every step."""
    gen = torch.Generator(device=device).manual_seed(seed)
    w = torch.ones(d, device=device) / d ** 0.5
    losses = [true_loss(w)]
    for _ in range(steps):
        G = worker_gradients(w, N, B, gen).contiguous()
        psi = aggregate(G)
        Hpsi = hessian_times(psi.double())
        eta = float(psi.double().dot(hessian_times(w.double())) / psi.double().dot(Hpsi))
        w = w - eta * psi
        losses.append(true_loss(w))
    return losses, w


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--workers", type=int, default=32)
    ap.add_argument("--batch", type=int, default=64)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--beta", type=float, default=0.99)
    args = ap.parse_args()
    import paper_2411_03742_amd as ada

    if not torch.cuda.is_available():
        print("this demo needs the GPU (the library has no CPU path)", file=sys.stderr)
        return 3
    d = 1000
    agg = ada.AdaCons(args.workers, d, beta=args.beta)
    out = torch.empty(d, device="cuda:0")
    mean_losses, _ = run(lambda G: G.mean(dim=0), args.workers, args.batch, args.steps)
    ada_losses, _ = run(lambda G: agg.aggregate(G, out=out).clone(), args.workers, args.batch, args.steps)
    print(f"N={args.workers} B={args.batch}: loss after {args.steps} steps  mean {mean_losses[-1]:.3e}   "
          f"AdaCons {ada_losses[-1]:.3e}   (start {mean_losses[0]:.3e})")
    for t in range(0, args.steps + 1, max(1, args.steps // 10)):
        print(f"  step {t:4d}   mean {mean_losses[t]:.4e}   AdaCons {ada_losses[t]:.4e}")
    agg.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
