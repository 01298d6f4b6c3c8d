"""Layer-wise aggregation: CPU checks of the oracle's composition, and GPU parity of the segmented
kernels against it."""
import numpy as np
import pytest
import torch

import workloads
from oracle import adacons_oracle as o

DEV = "cuda:0"


def _rand_layout(rng, d, L):
    cuts = np.sort(rng.choice(np.arange(1, d), size=L - 1, replace=False))
    return np.concatenate([[0], cuts, [d]]).astype(np.int64)


# ------------------------------------------------------------------ CPU: oracle composition ----
def test_single_layer_equals_model_wise():
    rng = np.random.default_rng(1)
    G = (rng.standard_normal(3000)[None, :] + 2 * rng.standard_normal((6, 3000))).astype(np.float32)
    out_m, info_m = o.aggregate(G, o.OracleState(6))
    out_l, infos = o.aggregate_layers(G, [0, 3000], [o.OracleState(6)])
    assert np.array_equal(out_m, out_l) and np.array_equal(info_m["gamma"], infos[0]["gamma"])


def test_layers_are_independent_and_keep_their_own_state():
    rng = np.random.default_rng(2)
    N, d = 5, 4000
    off = np.array([0, 7, 1000, 1001, 2500, d])
    states = [o.OracleState(N, beta=0.8) for _ in range(5)]
    ref_states = [o.OracleState(N, beta=0.8) for _ in range(5)]
    for t in range(4):
        G = (rng.standard_normal(d)[None, :] + 2 * rng.standard_normal((N, d))).astype(np.float32)
        out, infos = o.aggregate_layers(G, off, states)
        for l in range(5):
            a, b = off[l], off[l + 1]
            out_l, info_l = o.aggregate(np.ascontiguousarray(G[:, a:b]), ref_states[l])
            assert np.array_equal(out[a:b], out_l)
            assert np.array_equal(infos[l]["gamma"], info_l["gamma"])
            assert abs(infos[l]["gamma"].sum() - 1) < 1e-12
        # changing one layer's data leaves every other layer's weights alone
        G2 = G.copy(); G2[:, off[2]:off[3]] *= -3.0
        _, infos2 = o.aggregate_layers(G2, off, [o.OracleState(N, beta=0.8) for _ in range(5)])
        _, infos1 = o.aggregate_layers(G, off, [o.OracleState(N, beta=0.8) for _ in range(5)])
        for l in (0, 1, 3, 4):
            assert np.array_equal(infos1[l]["gamma"], infos2[l]["gamma"])


def test_resnet50_layout_adds_up():
    sizes = workloads.resnet50_layer_sizes()
    assert len(sizes) == 161 and sum(sizes) == workloads.C2.d and min(sizes) == 64


# --------------------------------------------------------------------------- GPU parity ----
@pytest.fixture(scope="module")
def pkg():
    if not torch.cuda.is_available():
        pytest.fail("these tests need the GPU")
    import paper_2411_03742_amd as p
    return p


def _ranks_unambiguous(raw, tol=1e-9):
    """The sort of Eq. 11 decides on floating-point values: parity of the per-worker assignment is
    only defined when no two coefficients are closer than the arithmetic error.  (A one-column
    layer is the extreme case: every a_i equals +-sum_j x_j / N in exact arithmetic.)"""
    s = np.sort(raw)
    return len(s) < 2 or np.diff(s).min() > tol * np.abs(s).max()


def _check_layers(pkg, G, off, agg, states, out_tol, check_out=True):
    out = agg.aggregate(G)
    info = agg.coeffs()
    Gh = workloads.to_oracle_input(G)
    first_step = states[0].t == 0
    oout, oinfos = o.aggregate_layers(Gh, off, states, want_out=check_out)
    mom = bool(states[0].flags & o.FLAG_MOMENTUM)
    for l, oi in enumerate(oinfos):
        assert info["numeric_flags"][l] == oi["numeric_flags"], l
        # from a zero state every rank receives (1 - beta) a_i: the assignment cannot matter yet
        strict = first_step or not mom or _ranks_unambiguous(oi["raw"])
        for key in ("gamma", "raw", "smoothed"):
            ref, got = oi[key], info[key][l]
            if not strict and key == "gamma":
                assert abs(got.sum() - 1.0) <= 1e-9
                continue
            if not strict and key == "smoothed":
                ref, got = np.sort(ref), np.sort(got)     # the same values, handed to tied workers in either order
            scale = np.maximum(np.abs(ref), 1e-3 * np.abs(ref).max() + 1e-300)
            assert (np.abs(got - ref) / scale).max() <= 1e-6, (l, key, got, ref)
        if check_out and not strict:
            # stage A3 is still checked: against the weighted sum of the weights the GPU chose
            a, b = off[l], off[l + 1]
            oout[a:b] = o.weighted_sum(np.ascontiguousarray(Gh[:, a:b]), info["gamma"][l])
    if check_out:
        got = out.cpu().numpy().astype(np.float64)
        assert np.linalg.norm(got - oout) / np.linalg.norm(oout) <= out_tol
        # every layer on its own as well (a small layer must not hide in the global norm), measured
        # against sum_i |gamma_i| |g_i|: what the rounding of an fp32 weighted sum is proportional to (a
        # layer of a few columns can cancel to a result far smaller than its terms)
        Gabs = G.float().abs().cpu().numpy().astype(np.float64)
        for l in range(len(oinfos)):
            a, b = off[l], off[l + 1]
            den = np.linalg.norm((np.abs(info["gamma"][l])[:, None] * Gabs[:, a:b]).sum(0))
            if den > 0:
                assert np.linalg.norm(got[a:b] - oout[a:b]) / den <= out_tol, l
    return out


@pytest.mark.gpu
@pytest.mark.parametrize("N,d,L", [(1, 64, 1), (2, 1000, 3), (4, 40_000, 17), (8, 300_000, 50), (8, 2_000_000, 9),
                                   (5, 123_456, 200), (8, 1024, 1024),
                                   (9, 50_000, 11), (16, 400_000, 40), (17, 1024, 1024), (33, 100_000, 7),
                                   (48, 60_000, 30), (64, 300_000, 25), (64, 64, 1),
                                   (65, 30_000, 9), (80, 200_000, 20), (100, 50_000, 50), (128, 150_000, 12), (128, 1024, 64)])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_random_layouts_match_oracle(pkg, N, d, L, dtype):
    rng = np.random.default_rng(N * 7 + L)
    vec = 8 if dtype == torch.bfloat16 else 4
    d = (d + vec - 1) // vec * vec
    off = _rand_layout(rng, d, L) if L < d else np.arange(d + 1, dtype=np.int64)
    g = torch.Generator(device=DEV).manual_seed(L)
    agg = pkg.AdaConsLayers(N, off, dtype=dtype, beta=0.9)
    states = [o.OracleState(N, beta=0.9) for _ in range(len(off) - 1)]
    for t in range(3):
        s = torch.randn(d, generator=g, device=DEV)
        G = (s[None, :] + 2.0 * torch.randn(N, d, generator=g, device=DEV)).to(dtype).contiguous()
        _check_layers(pkg, G, off, agg, states, 1e-5 if dtype == torch.float32 else 2e-3)
    agg.close()


@pytest.mark.gpu
@pytest.mark.parametrize("N,d,L,shift", [(2, 1001, 3, 0), (4, 40_003, 17, 1), (8, 300_005, 50, 0), (8, 9, 2, 0), (5, 123_457, 200, 3),
                                         (8, 1027, 1027, 0), (9, 50_001, 11, 1), (16, 400_006, 40, 0), (33, 100_007, 7, 5),
                                         (64, 300_002, 25, 0), (64, 71, 1, 1), (8, 300_000, 50, 2),
                                         (97, 60_003, 13, 1), (128, 40_001, 5, 0)])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_layouts_off_the_16_byte_grid(pkg, N, d, L, shift, dtype):
    """d that is not a multiple of the 128-bit group (the last group of every row is ragged), G and out
    starting `shift` elements past a 16-byte boundary: same parity bar as the aligned layouts."""
    rng = np.random.default_rng(N * 11 + L)
    off = _rand_layout(rng, d, L) if L < d else np.arange(d + 1, dtype=np.int64)
    g = torch.Generator(device=DEV).manual_seed(L + 1)
    agg = pkg.AdaConsLayers(N, off, dtype=dtype, beta=0.9)
    states = [o.OracleState(N, beta=0.9) for _ in range(len(off) - 1)]
    buf = torch.empty(N * d + shift, device=DEV, dtype=dtype)
    G = buf[shift:].view(N, d)
    assert G.is_contiguous()
    for t in range(2):
        s = torch.randn(d, generator=g, device=DEV)
        G.copy_((s[None, :] + 2.0 * torch.randn(N, d, generator=g, device=DEV)).to(dtype))
        _check_layers(pkg, G, off, agg, states, 1e-5 if dtype == torch.float32 else 2e-3)
    # an output that starts off the 16-byte grid, with guard elements on both sides
    obuf = torch.full((d + 2,), 7.0, device=DEV)
    agg2 = pkg.AdaConsLayers(N, off, dtype=dtype, beta=0.9, flags=0)   # no momentum: same input, same output
    a = agg2.aggregate(G).clone()
    b = agg2.aggregate(G, out=obuf[1:d + 1])
    assert torch.equal(a, b) and obuf[0] == 7.0 and obuf[d + 1] == 7.0
    agg.close(); agg2.close()


@pytest.mark.gpu
@pytest.mark.parametrize("N,L", [(12, 40), (16, 161)])
def test_long_fp32_streams_of_many_workers(pkg, N, L):
    """fp32, N >= 12, d >= 2^24: the second pass parks whole pieces of output in LDS and writes them in
    bursts; pieces on layer boundaries and at the ragged end of a row take the masked path."""
    d = (1 << 24) + 12_345
    rng = np.random.default_rng(L)
    off = _rand_layout(rng, d, L)
    g = torch.Generator(device=DEV).manual_seed(N)
    agg = pkg.AdaConsLayers(N, off, beta=0.9)
    states = [o.OracleState(N, beta=0.9) for _ in range(L)]
    for t in range(2):
        s = torch.randn(d, generator=g, device=DEV)
        G = (s[None, :] + 2.0 * torch.randn(N, d, generator=g, device=DEV)).contiguous()
        _check_layers(pkg, G, off, agg, states, 1e-5)
    agg.close()


@pytest.mark.gpu
def test_layers_need_one_whole_group(pkg):
    with pytest.raises(pkg.AdaConsError) as e:
        pkg.AdaConsLayers(4, [0, 2, 3])
    assert e.value.status == 1


@pytest.mark.gpu
def test_resnet50_layout_full_size(pkg):
    """C2's shape (N = 8, d = 25,557,032, fp32) cut into the 161 parameter tensors of a ResNet-50;
    three steps of the C2 stream with momentum."""
    w = workloads.C2.scaled(workloads.C2.d, 3)
    off = np.concatenate([[0], np.cumsum(workloads.resnet50_layer_sizes())]).astype(np.int64)
    agg = pkg.AdaConsLayers(w.N, off, beta=0.99)
    states = [o.OracleState(w.N, beta=0.99) for _ in range(len(off) - 1)]
    for t, G in enumerate(workloads.stream(w, DEV)):
        _check_layers(pkg, G, off, agg, states, 1e-5, check_out=(t == 2))
    agg.close()


@pytest.mark.gpu
def test_one_layer_equals_model_wise_kernel(pkg):
    N, d = 8, 1_000_000
    g = torch.Generator(device=DEV).manual_seed(5)
    G = (torch.randn(d, generator=g, device=DEV)[None, :] + torch.randn(N, d, generator=g, device=DEV)).contiguous()
    a = pkg.AdaCons(N, d)
    b = pkg.AdaConsLayers(N, [0, d])
    oa, ob = a.aggregate(G), b.aggregate(G)
    ga, gb = a.coeffs()["gamma"], b.coeffs()["gamma"][0]
    assert np.abs(ga - gb).max() <= 1e-12 * np.abs(ga).max()
    assert torch.allclose(oa, ob, rtol=1e-6, atol=1e-7)
    a.close(); b.close()


@pytest.mark.gpu
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_one_layer_equals_model_wise_kernel_many_workers(pkg, dtype):
    """N > 8: the per-layer statistics against the model-wise path (Gram on the matrix cores)."""
    N, d = 32, 500_000
    g = torch.Generator(device=DEV).manual_seed(6)
    G = (torch.randn(d, generator=g, device=DEV)[None, :] + 2 * torch.randn(N, d, generator=g, device=DEV)).to(dtype).contiguous()
    a = pkg.AdaCons(N, d)
    b = pkg.AdaConsLayers(N, [0, d], dtype=dtype)
    oa, ob = a.aggregate(G), b.aggregate(G)
    ga, gb = a.coeffs()["gamma"], b.coeffs()["gamma"][0]
    assert np.abs(ga - gb).max() <= 1e-6 * np.abs(ga).max()
    assert torch.allclose(oa, ob, rtol=1e-4, atol=1e-5)
    a.close(); b.close()


@pytest.mark.gpu
def test_layer_argument_errors(pkg):
    with pytest.raises(pkg.AdaConsError) as e:
        pkg.AdaConsLayers(129, [0, 100])
    assert e.value.status == 2
    with pytest.raises(pkg.AdaConsError):
        pkg.AdaConsLayers(4, [0, 50, 50, 100])          # empty layer
    with pytest.raises(pkg.AdaConsError):
        pkg.AdaConsLayers(4, [1, 100])
    agg = pkg.AdaConsLayers(4, [0, 40, 100])
    with pytest.raises(pkg.AdaConsError):
        agg.aggregate(torch.zeros(4, 104, device=DEV))  # d differs from the layout
    agg.close()
