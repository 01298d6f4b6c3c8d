"""One worker's share of Algorithm 1: pair statistics, coefficient update from gathered statistics,
in-place rescaling.  CPU pins of the oracle side, GPU parity of the kernels."""
import numpy as np
import pytest
import torch

import workloads
from oracle import adacons_oracle as o

DEV = "cuda:0"


# ----------------------------------------------------------------------------- CPU pins ----
def test_coefficients_from_stats_equal_coefficients_from_gram():
    """O2 only reads the diagonal and the row sums of K: feeding those directly gives the same
    weights, bit for bit, and the same state."""
    rng = np.random.default_rng(11)
    N, d = 9, 500
    s1, s2 = o.OracleState(N, beta=0.8), o.OracleState(N, beta=0.8)
    for _ in range(5):
        G = (rng.standard_normal(d)[None, :] + 2 * rng.standard_normal((N, d))).astype(np.float32)
        K = o.gram(G)
        a = o.coefficients(K, s1)
        b = o.coefficients_from_stats(np.diag(K).copy(), np.array([K[i].cumsum()[-1] for i in range(N)]), s2)
        r_seq = np.array([sum(K[i, j] for j in range(N)) for i in range(N)])      # j ascending, like O2
        assert np.array_equal(r_seq, np.array([K[i].cumsum()[-1] for i in range(N)]))
        for key in ("gamma", "raw", "smoothed"):
            assert np.array_equal(a[key], b[key])
        assert np.array_equal(s1.m, s2.m) and s1.t == s2.t


def test_worker_stats_are_the_dot_products_of_algorithm_1():
    rng = np.random.default_rng(12)
    N, d = 6, 70_001
    G = (rng.standard_normal(d)[None, :] + rng.standard_normal((N, d))).astype(np.float32)
    gsum = G.astype(np.float64).sum(0).astype(np.float32)        # the all-reduced sum, as stored
    for i in range(N):
        sq, dot, ss = o.worker_stats(G[i], gsum)
        g64, s64 = G[i].astype(np.float64), gsum.astype(np.float64)
        assert np.isclose(sq, g64 @ g64, rtol=1e-13) and np.isclose(dot, g64 @ s64, rtol=1e-12)
        assert np.isclose(ss, s64 @ s64, rtol=1e-13)


def test_algorithm_1_route_agrees_with_the_gram_route():
    """<g_i, fp32(sum g)> differs from sum_j K_ij only by the rounding of the stored sum."""
    rng = np.random.default_rng(13)
    N, d = 8, 200_000
    G = (rng.standard_normal(d)[None, :] + 2 * rng.standard_normal((N, d))).astype(np.float32)
    gsum = G.astype(np.float64).sum(0).astype(np.float32)
    stats = [o.worker_stats(G[i], gsum) for i in range(N)]
    a = o.coefficients_from_stats([s[0] for s in stats], [s[1] for s in stats], o.OracleState(N))
    _, b = o.aggregate(G, o.OracleState(N), want_out=False)
    assert np.allclose(a["gamma"], b["gamma"], rtol=1e-6)


# --------------------------------------------------------------------------- GPU parity ----
@pytest.fixture(scope="module")
def pkg():
    if not torch.cuda.is_available():
        pytest.fail("these tests need the GPU")
    import paper_2411_03742_amd as p
    return p


def _bits(t):
    return workloads.to_oracle_input(t.reshape(1, -1))[0]


@pytest.mark.gpu
@pytest.mark.parametrize("d", [1, 5, 4096, 100_003, 1_048_576 + 8, 25_557_032])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_worker_stats_match_oracle(pkg, d, dtype):
    g = torch.Generator(device=DEV).manual_seed(d % 1000)
    x = torch.randn(d, generator=g, device=DEV).to(dtype)
    y = (3.0 * torch.randn(d, generator=g, device=DEV) + x.float()).to(dtype)
    agg = pkg.AdaCons(4, d)
    got = agg.worker_stats(x, y).cpu().numpy()
    ref = np.array(o.worker_stats(_bits(x), _bits(y)))
    scale = np.array([ref[0], np.sqrt(ref[0] * ref[2]), ref[2]])
    assert (np.abs(got - ref) / scale).max() <= 1e-12
    same = agg.worker_stats(x, x).cpu().numpy()
    assert same[0] == same[1] == same[2]
    agg.close()


@pytest.mark.gpu
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("d", [1, 3, 7, 9, 50_000, 50_001, 50_003, 50_005, 50_007, 262_150])
@pytest.mark.parametrize("shift", [0, 1])
def test_worker_stats_and_scale_off_16_byte_boundaries(pkg, d, dtype, shift):
    """Vectors that start one element past a 16-byte boundary and lengths with every leftover count:
    the 128-bit kernels run from element-aligned addresses, the leftover elements go to single threads."""
    buf = torch.randn(2 * d + 2 * shift + 8, device=DEV).to(dtype)
    x, y = buf[shift:d + shift], buf[d + shift:2 * d + shift]
    agg = pkg.AdaCons(2, d, flags=0)
    got = agg.worker_stats(x, y).cpu().numpy()
    ref = np.array(o.worker_stats(_bits(x), _bits(y)))
    assert np.allclose(got, ref, rtol=1e-12)
    # the weights the scale uses: with momentum and normalisation off gamma_i = r_i / (N q_i) = 0.75, -1.25 exactly
    agg.update_from_stats([1.0, 1.0], [1.5, -2.5])
    assert np.array_equal(agg.coeffs()["gamma"], [0.75, -1.25])
    before = buf.clone()
    agg.worker_scale(x, 1)
    want = (before[shift:d + shift].float() * (-1.25)).to(dtype)
    assert torch.equal(x.view(torch.int16 if dtype == torch.bfloat16 else torch.int32),
                       want.view(torch.int16 if dtype == torch.bfloat16 else torch.int32))
    # nothing outside the vector was touched
    assert torch.equal(buf[:shift], before[:shift]) and torch.equal(buf[d + shift:], before[d + shift:])
    agg.close()


@pytest.mark.gpu
@pytest.mark.parametrize("N,d,dtype", [(8, 1_000_004, torch.float32), (16, 200_000, torch.float32),
                                       (5, 77_777, torch.float32), (8, 400_008, torch.bfloat16),
                                       (128, 30_000, torch.float32)])
def test_algorithm_1_on_one_gpu(pkg, N, d, dtype):
    """Every step of Algorithm 1 with the collectives replaced by what they would deliver: the sum of
    the gradients (step 1), the gathered pairs (step 2); then the coefficient update (step 3), the
    per-worker rescaling and the final sum (step 4).  Checked against the oracle fed with the same
    stored sum, and against the single-call Gram route."""
    agg = pkg.AdaCons(N, d, beta=0.9)
    ref_agg = pkg.AdaCons(N, d, beta=0.9)
    ost = o.OracleState(N, beta=0.9)
    gen = torch.Generator(device=DEV).manual_seed(N + d % 997)
    for t in range(3):
        s = torch.randn(d, generator=gen, device=DEV)
        G = (s[None, :] + 2.0 * torch.randn(N, d, generator=gen, device=DEV)).to(dtype).contiguous()
        gsum = G.float().sum(0).to(dtype)                        # what the all-reduce leaves on every worker
        stats = torch.stack([agg.worker_stats(G[i], gsum) for i in range(N)]).cpu().numpy()
        agg.update_from_stats(stats[:, 0], stats[:, 1])
        info = agg.coeffs()
        ostats = [o.worker_stats(_bits(G[i]), _bits(gsum)) for i in range(N)]
        oinfo = o.coefficients_from_stats([x[0] for x in ostats], [x[1] for x in ostats], ost)
        assert info["numeric_flags"] == oinfo["numeric_flags"] == 0
        for key in ("gamma", "raw", "smoothed"):
            assert (np.abs(info[key] - oinfo[key]) / np.abs(oinfo[key])).max() <= 1e-9, key
        # step 4: rescale in place, then the sum the final all-reduce would form
        scaled = G.clone()
        for i in range(N):
            agg.worker_scale(scaled[i], i)
        g32 = info["gamma"].astype(np.float32)
        for i in (0, N - 1):
            ref_i = o.weighted_sum(_bits(G[i]).reshape(1, -1), [float(g32[i])])
            got_i = scaled[i].float().cpu().numpy()
            tol = 1e-6 if dtype == torch.float32 else 4e-3
            assert np.linalg.norm(got_i - ref_i) / np.linalg.norm(ref_i) <= tol
            if dtype == torch.bfloat16:                          # rounding is round-to-nearest-even
                lib = (G[i].float() * float(g32[i])).to(torch.bfloat16)
                assert torch.equal(lib.view(torch.int16), scaled[i].view(torch.int16))
        total = scaled.float().sum(0).cpu().numpy()
        # the single-call route on the same gradients
        out = ref_agg.aggregate(G).cpu().numpy()
        gam_ref = ref_agg.coeffs()["gamma"]
        assert (np.abs(info["gamma"] - gam_ref) / np.abs(gam_ref)).max() <= (5e-6 if dtype == torch.float32 else 2e-2)
        tol = 1e-5 if dtype == torch.float32 else 2e-2
        assert np.linalg.norm(total - out) / np.linalg.norm(out) <= tol
    agg.close(); ref_agg.close()


@pytest.mark.gpu
def test_worker_share_argument_errors(pkg):
    agg = pkg.AdaCons(4, 100)
    x = torch.randn(100, device=DEV)
    with pytest.raises(pkg.AdaConsError):
        agg.worker_scale(x, 4)
    with pytest.raises(pkg.AdaConsError):
        agg.worker_stats(torch.randn(101, device=DEV), torch.randn(101, device=DEV))   # d > d_max
    agg.close()
