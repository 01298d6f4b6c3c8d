"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.

The oracle computes the whole float64 Gram matrix and coefficients for these inputs (seconds on
the host's cores); the d-length output is compared on sampled columns, which the oracle evaluates
one by one: the first and last 256 columns (tile heads and ragged tails) and 8192 seeded random
ones.  Multi-step configurations run a prefix of their step count here; the whole step count runs
at reduced length in test_parity_gpu.py.
"""
import numpy as np
import pytest
import torch

import workloads
from oracle import adacons_oracle as o

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
OUT_TOL = {"f32": 1e-5, "bf16": 2e-3}


@pytest.fixture(scope="module")
def pkg():
    if not torch.cuda.is_available():
        pytest.fail("these tests need the GPU")
    import paper_2411_03742_amd as p
    return p


def sample_columns(d, seed):
    rng = np.random.default_rng(seed)
    edge = min(256, d)
    idx = np.concatenate([np.arange(edge), np.arange(d - edge, d), rng.integers(0, d, 8192)])
    return np.unique(idx)


@pytest.mark.parametrize("name,steps,stats_only", [("C2", 20, 0), ("C3", 1, 0), ("C4", 2, 0), ("C5", 3, 0),
                                                   ("C4", 2, 1), ("C5", 2, 1), ("C4-bf16", 2, 0)])
def test_full_size_configuration(pkg, name, steps, stats_only):
    if name == "C4-bf16":     # C4's shape and recipe stored as bf16: the bf16 matrix-core Gram at full length
        from dataclasses import replace
        w = replace(workloads.C4, name="C4-bf16", dtype="bf16")
    else:
        w = workloads.CONFIGS[name]
    w = w.scaled(w.d, steps)
    agg = pkg.AdaCons(w.N, w.d, beta=0.99)
    agg.tune(pkg.ADACONS_TUNE_STATS_ONLY, stats_only)   # 1: stage A1 computes diag K and row sums only
    ost = o.OracleState(w.N, beta=0.99)
    out = torch.empty(w.d, dtype=torch.float32, device=DEV)
    for t, G in enumerate(workloads.stream(w, DEV)):
        agg.aggregate(G, out=out)
        info = agg.coeffs()
        Gh = workloads.to_oracle_input(G)
        _, oinfo = o.aggregate(Gh, ost, want_out=False)
        assert info["numeric_flags"] == oinfo["numeric_flags"] == 0
        s = np.sort(oinfo["raw"])
        assert np.diff(s).min() > 1e-9 * np.abs(s).max()           # ranks are unambiguous
        for key in ("gamma", "raw", "smoothed"):
            ref = oinfo[key]
            assert np.linalg.norm(info[key] - ref) / np.linalg.norm(ref) <= 1e-6, (name, t, key)
            assert (np.abs(info[key] - ref) / np.abs(ref)).max() <= 1e-6, (name, t, key)
        idx = sample_columns(w.d, seed=t)
        ref = o.weighted_sum_at(Gh, oinfo["gamma"], idx)
        got = out[torch.from_numpy(idx).to(DEV)].cpu().numpy().astype(np.float64)
        assert np.linalg.norm(got - ref) / np.linalg.norm(ref) <= OUT_TOL[w.dtype], (name, t)
        # every element was written: the output of an all-positive-weight step cannot keep the
        # poison the buffer is refilled with below
        assert torch.isfinite(out).all()
        out.fill_(float("nan"))
        del Gh
    agg.close()
