"""GPU parity: the HIP path (through the C ABI) against the float64 CPU oracle, element by element,
on the same seeded inputs.  Sizes here are ones the oracle finishes in seconds, spanning several
tiles and ragged tails; full-size configurations live in test_full_size_gpu.py.

Tolerances (stated by the benchmark definition): out relative L2 error <= 1e-5 for fp32 inputs and
<= 2e-3 for bf16 inputs; coefficients <= 1e-6 relative.
"""
import numpy as np
import pytest
import torch

import workloads
from oracle import adacons_oracle as o

pytestmark = pytest.mark.gpu

OUT_TOL = {torch.float32: 1e-5, torch.bfloat16: 2e-3}
GAMMA_TOL = 1e-6
DEV = "cuda:0"


@pytest.fixture(scope="module")
def pkg():
    if not torch.cuda.is_available():
        pytest.fail("these tests need the GPU")
    import paper_2411_03742_amd as p
    return p


from parity_checks import (assert_out_elementwise, assert_vec_close, check_coefficients, check_out, rel_l2)


def assert_gamma_close(got, ref, tol=GAMMA_TOL):
    assert_vec_close(got, ref, tol)


def randG(N, d, dtype=torch.float32, sigma=1.0, seed=0):
    g = torch.Generator(device=DEV).manual_seed(seed)
    s = torch.randn(d, generator=g, device=DEV)
    G = s[None, :] + sigma * torch.randn(N, d, generator=g, device=DEV)
    return G.to(dtype).contiguous()


def both(pkg, G, agg, ost, check_output=True, ties_possible=False):
    """One aggregation on both sides.  Coefficients are compared one to one whenever the two sides
    sorted alike (asserted unless ties_possible: one-column inputs, where every a_i is +-sum x / N);
    `out` is held to the element-wise rounding bound against the oracle's weighted sum of the weights
    the GPU applied, and to the stated relative L2 tolerance against the oracle's own output.
    Returns (out, info, oinfo); oinfo["strict"] says whether the comparison was one to one."""
    state_was_zero = not ost.m.any()
    out = agg.aggregate(G)
    info = agg.coeffs()
    Gh = workloads.to_oracle_input(G)
    oout, oinfo = o.aggregate(Gh, ost, want_out=check_output)
    strict = check_coefficients(info, oinfo, ost.m, ost.flags, state_was_zero, ties_possible)
    oinfo["strict"] = strict
    if check_output and not (oinfo["numeric_flags"] & o.NUM_NONFINITE):
        check_out(out.cpu().numpy(), Gh, info, oout, strict)
    return out, info, oinfo


# ------------------------------------------------------------------------------ stage A1 ----
GRAM_SHAPES = [(1, 1), (1, 1000), (2, 5), (3, 4096), (4, 100_003), (5, 262_144 + 64), (7, 33_333),
               (8, 1_048_576 + 4), (8, 1023), (9, 70_000), (16, 200_000), (16, 17), (17, 50_001),
               (32, 65_536 + 12), (33, 10_000), (48, 30_000), (63, 9_999), (64, 131_072 + 20)]


@pytest.mark.parametrize("N,d", GRAM_SHAPES)
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_gram_matches_oracle(pkg, N, d, dtype):
    G = randG(N, d, dtype, sigma=2.0, seed=N * 1000 + d % 997)
    agg = pkg.AdaCons(N, d)
    K = agg.gram(G)
    Kref = o.gram(workloads.to_oracle_input(G))
    scale = np.sqrt(np.outer(np.diag(Kref), np.diag(Kref)))
    # N <= 8 accumulates in fp64; larger N sums 128 fp32 products on the matrix cores between
    # fp64 flushes
    tol = 1e-12 if N <= 8 else 3e-7
    assert (np.abs(K - Kref) / scale).max() <= tol
    assert np.array_equal(K, K.T)
    agg.close()


@pytest.mark.parametrize("N,d", [(12, 1024), (16, 4096 + 16), (24, 100_000), (40, 20_000), (64, 65_536 + 256)])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("variant", [0, 1])
def test_gram_matrix_core_variants_match_oracle(pkg, N, d, dtype, variant):
    """The two matrix-core Gram kernels, each at every tile count: products on the fp32 instruction (0),
    and every fp32 product formed from six exact bf16 products (1)."""
    G = randG(N, d, dtype, sigma=2.0, seed=N + d % 991)
    agg = pkg.AdaCons(N, d)
    agg.tune(pkg.ADACONS_TUNE_GRAM_PRODUCTS, variant)
    K = agg.gram(G)
    Kref = o.gram(workloads.to_oracle_input(G))
    scale = np.sqrt(np.outer(np.diag(Kref), np.diag(Kref)))
    assert (np.abs(K - Kref) / scale).max() <= 3e-7
    agg.close()


def test_gram_distinct_rows_exact(pkg):
    """Small integers: every product and sum is exact in any precision, so a transposed tile or a
    wrong row/column mapping shows as an exact mismatch."""
    for N, d in [(3, 5), (8, 64), (16, 40), (40, 100), (64, 257)]:
        G = ((torch.arange(N * d, device=DEV) * 7 + 3) % 11 - 5).float().reshape(N, d).contiguous()
        agg = pkg.AdaCons(N, d)
        K = agg.gram(G)
        G64 = G.cpu().numpy().astype(np.float64)
        assert np.array_equal(K, G64 @ G64.T), (N, d)
        assert np.array_equal(K, o.gram(G.cpu().numpy()))
        agg.close()


# ------------------------------------------------------------------------------ stage A3 ----
@pytest.mark.parametrize("N,d", [(1, 7), (4, 1_048_576), (8, 100_003), (8, 2_097_152 + 8), (13, 50_000),
                                 (16, 300_000), (64, 70_004)])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_weighted_sum_with_given_weights(pkg, N, d, dtype):
    G = randG(N, d, dtype, sigma=1.5, seed=d % 1009)
    gamma = np.random.default_rng(N).standard_normal(N) / N
    agg = pkg.AdaCons(N, d)
    out = agg.weighted_sum(G, gamma).cpu().numpy()
    ref = o.weighted_sum(workloads.to_oracle_input(G), gamma.astype(np.float32).astype(np.float64))
    assert rel_l2(out, ref) <= 1e-6
    ref64 = o.weighted_sum(workloads.to_oracle_input(G), gamma)
    assert rel_l2(out, ref64) <= OUT_TOL[dtype]
    assert_out_elementwise(out, workloads.to_oracle_input(G), gamma)
    agg.close()


def test_weighted_sum_leaves_the_reported_coefficients_alone(pkg):
    """Stage A3 with the caller's weights uses a buffer of its own: adacons_coeffs still reports the
    last aggregation, and the next aggregation is not disturbed."""
    N, d = 8, 100_000
    G = randG(N, d, sigma=2.0, seed=4)
    agg = pkg.AdaCons(N, d, beta=0.9)
    ref = pkg.AdaCons(N, d, beta=0.9)
    agg.aggregate(G); ref.aggregate(G)
    before = agg.coeffs()
    agg.weighted_sum(G, np.linspace(-1.0, 2.0, N))
    after = agg.coeffs()
    for key in ("gamma", "raw", "smoothed"):
        assert np.array_equal(before[key], after[key])
    G2 = randG(N, d, sigma=2.0, seed=5)
    assert torch.equal(agg.aggregate(G2), ref.aggregate(G2))
    agg.close(); ref.close()


@pytest.mark.parametrize("N,d", [(9, 1000), (13, 5003), (16, 1000), (17, 1001), (24, 4100), (33, 70_003), (64, 3), (100, 8), (128, 1000),
                                 (128, 65_536 + 24), (48, 300_000)])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_weighted_sum_by_row_slices(pkg, N, d, dtype):
    """Stage A3 for many workers with few parameters each: the rows shared out over the wavefronts of a
    workgroup (ADACONS_TUNE_WSUM_ROW_SLICES = 2 forces it for N > 8), partial sums added in wavefront
    order.  Every element within the rounding bound of an fp32 sum of N terms; the descent step likewise."""
    G = randG(N, d, dtype, sigma=1.5, seed=d % 1009 + N)
    Gh = workloads.to_oracle_input(G)
    gamma = np.random.default_rng(N).standard_normal(N) / N
    agg = pkg.AdaCons(N, d)
    agg.tune(pkg.ADACONS_TUNE_WSUM_ROW_SLICES, 2)
    out = torch.full((d,), float("nan"), device=DEV)
    out = agg.weighted_sum(G, gamma, out=out).cpu().numpy()
    assert_out_elementwise(out, Gh, gamma)
    assert rel_l2(out, o.weighted_sum(Gh, gamma)) <= OUT_TOL[dtype]
    # whole aggregation and the fused step through the same kernel (the coefficients of a handful of columns
    # are too ill-conditioned for the stated tolerance, whatever the kernel: only the sums are checked there)
    agg.aggregate(G) if d < 512 else both(pkg, G, agg, o.OracleState(N))
    w = torch.randn(d, device=DEV)
    w0 = w.cpu().numpy()
    agg.aggregate_apply(G, w, lr=0.25)
    assert_out_elementwise(w.cpu().numpy(), Gh, agg.coeffs()["gamma"], base=w0, lr=0.25)
    agg.close()


def test_row_slices_are_the_default_for_many_workers_and_short_gradients_only(pkg):
    """Default choice of the stage A3 kernel: the two kernels add in different orders, so their outputs
    differ in the last bits; the default must equal the forced row slices for N > 16 at up to 256 column
    groups per CU and for N > 8 at up to 1 MiB of gradients, and the column kernel elsewhere."""
    for N, d, rows in [(32, 1000, True), (128, 8192, True), (17, 65_536, True), (16, 1000, True), (16, 65_536, False),
                       (8, 1000, False), (32, 1 << 20, False)]:
        G = randG(N, d, seed=3)
        outs = []
        for mode in (1, 2, 0):
            agg = pkg.AdaCons(N, d)
            agg.tune(pkg.ADACONS_TUNE_WSUM_ROW_SLICES, mode)
            outs.append(agg.aggregate(G).clone())
            agg.close()
        if N > 8:
            assert not torch.equal(outs[1], outs[2])       # the inputs do tell the two kernels apart
        assert torch.equal(outs[0], outs[1] if rows else outs[2]), (N, d)


# --------------------------------------------------------------------- whole aggregation ----
@pytest.mark.parametrize("name,d,steps", [("C1", None, 1), ("C2", 1_048_576 + 40, 20), ("C3", 2_097_152 + 3072, 1),
                                          ("C4", 262_144 + 8, 10), ("C5", 524_288 + 64, 100)])
def test_config_streams_at_test_size(pkg, name, d, steps):
    """The five benchmark recipes (same N, dtype, value distribution, step count) at a length the
    oracle handles in seconds; coefficients checked at every step, outputs at every step."""
    w = workloads.CONFIGS[name]
    w = w if d is None else w.scaled(d, steps)
    agg = pkg.AdaCons(w.N, w.d, beta=0.99)
    ost = o.OracleState(w.N, beta=0.99)
    for t, G in enumerate(workloads.stream(w, DEV)):
        _, info, oinfo = both(pkg, G, agg, ost, check_output=(t % 10 == 0 or t == steps - 1))
        assert oinfo["strict"]               # continuous inputs: both sides sort alike at every step
        assert abs(info["gamma"].sum() - 1.0) <= 1e-9
        if name == "C5":
            assert info["gamma"].min() < 0 and (info["gamma"] > 0).sum() == w.N - 1
    m, step = agg.export_state()
    assert step == steps
    assert_gamma_close(m, ost.m)
    agg.close()


@pytest.mark.parametrize("flags", [0, 1, 2, 3, 5, 7, 10, 11, 15])
@pytest.mark.parametrize("N", [5, 8, 16])
def test_ablation_variants(pkg, flags, N):
    """The four columns of Table 2 (momentum and normalisation on/off), and the two variants:
    +4 the index-coupled EMA of Eq. 10, +8 lambda as Eq. 13 prints it."""
    d = 150_000
    agg = pkg.AdaCons(N, d, beta=0.9, flags=flags)
    ost = o.OracleState(N, beta=0.9, flags=flags)
    for t in range(4):
        G = randG(N, d, sigma=2.0, seed=100 + t)
        if flags & 4:
            G = G[torch.roll(torch.arange(N), t).to(DEV)].contiguous()   # worker order matters for Eq. 10
        both(pkg, G, agg, ost)
    m, _ = agg.export_state()
    assert np.allclose(m, ost.m, rtol=1e-6, atol=1e-12)
    agg.close()


def test_identical_gradients_reduce_to_averaging(pkg):
    N, d = 8, 500_000
    g = torch.randn(d, device=DEV)
    G = g[None, :].repeat(N, 1).contiguous()
    agg = pkg.AdaCons(N, d)
    out = agg.aggregate(G)
    info = agg.coeffs()
    assert np.allclose(info["gamma"], 1.0 / N, rtol=1e-12)
    assert rel_l2(out.cpu().numpy(), g.cpu().numpy()) <= 1e-6
    agg.close()


def test_permuting_workers_permutes_weights_only(pkg):
    N, d, T = 16, 200_000, 6
    a1, a2 = pkg.AdaCons(N, d, beta=0.9), pkg.AdaCons(N, d, beta=0.9)
    rng = np.random.default_rng(5)
    for t in range(T):
        G = randG(N, d, sigma=2.0, seed=40 + t)
        perm = torch.from_numpy(rng.permutation(N)).to(DEV)
        o1, o2 = a1.aggregate(G), a2.aggregate(G.index_select(0, perm).contiguous())
        g1, g2 = a1.coeffs()["gamma"], a2.coeffs()["gamma"]
        assert_gamma_close(g2, g1[perm.cpu().numpy()], 1e-9)
        assert rel_l2(o2.cpu().numpy(), o1.cpu().numpy()) <= 1e-6
    a1.close(); a2.close()


def test_runs_are_bit_identical(pkg):
    N, d = 8, 3_000_000
    G = randG(N, d, seed=9)
    outs, gams = [], []
    for _ in range(3):
        agg = pkg.AdaCons(N, d)
        outs.append(agg.aggregate(G).clone())
        gams.append(agg.coeffs()["gamma"])
        agg.close()
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])
    assert np.array_equal(gams[0], gams[1]) and np.array_equal(gams[0], gams[2])


@pytest.mark.parametrize("N,d,dtype,flags", [(4, 1 << 20, torch.float32, 3), (8, 500_000, torch.float32, 3),
                                             (8, 400_008, torch.bfloat16, 3), (1, 4096, torch.float32, 3),
                                             (5, 100_004, torch.float32, 0), (7, 33_336, torch.bfloat16, 7),
                                             (2, 8, torch.float32, 11), (3, 2_000_004, torch.float32, 1)])
def test_short_path_equals_three_launches_bit_for_bit(pkg, N, d, dtype, flags):
    """ADACONS_TUNE_SHORT_PATH: stage A2 inside stage A3 (two launches, the momentum state double-buffered)
    against the three-launch path on the same stream of inputs: output, coefficients, K and the carried
    state must be equal bit for bit -- over regular steps, a zero row, a non-finite step (state left
    untouched) and a regular step after it -- and the fused descent step likewise."""
    short_against_plain(pkg, N, d, dtype, flags, 0)


@pytest.mark.parametrize("N,d,dtype,flags,stats_only", [
    (9, 1000, torch.float32, 3, 0), (12, 4096, torch.bfloat16, 3, 0), (16, 16384, torch.float32, 3, 0), (16, 1000, torch.float32, 3, 1),
    (17, 1000, torch.float32, 3, 0), (32, 1000, torch.float32, 3, 0), (44, 2048, torch.float32, 7, 0),
    (32, 8192, torch.float32, 3, 0),     # 1 MiB: the cap on stage A1's partial rows binds
    (24, 1008, torch.bfloat16, 3, 0), (40, 512, torch.float32, 0, 0),
    (64, 1000, torch.float32, 3, 1), (20, 5000, torch.float32, 11, 1), (48, 2000, torch.bfloat16, 3, 1),
    (65, 1000, torch.float32, 3, 0), (100, 1000, torch.float32, 3, 0), (128, 1000, torch.float32, 7, 0),
    (128, 2048, torch.float32, 3, 0), (128, 1000, torch.bfloat16, 3, 0)])
def test_short_path_for_many_workers_equals_three_launches_bit_for_bit(pkg, N, d, dtype, flags, stats_only):
    """The same for N > 8 at up to 1 MiB of gradients (many workers with few parameters each, the regime of
    Eq. 14's example), where stage A3 runs by row slices: packed Gram rows for N <= 44, the rows of the
    statistics-only pass (chosen, or N > 64) for any N."""
    short_against_plain(pkg, N, d, dtype, flags, stats_only)


def short_against_plain(pkg, N, d, dtype, flags, stats_only):
    short, plain = pkg.AdaCons(N, d, beta=0.9, flags=flags), pkg.AdaCons(N, d, beta=0.9, flags=flags)
    short.tune(pkg.ADACONS_TUNE_SHORT_PATH, 2)
    plain.tune(pkg.ADACONS_TUNE_SHORT_PATH, 0)
    short.tune(pkg.ADACONS_TUNE_STATS_ONLY, stats_only)
    plain.tune(pkg.ADACONS_TUNE_STATS_ONLY, stats_only)
    has_K = N <= 64 and not (stats_only and N > 8)
    # two launches on one side, three on the other: seen through the per-stage timing
    G = randG(N, d, dtype, sigma=2.0, seed=899)
    for two in (True, False):
        probe = pkg.AdaCons(N, d)
        probe.tune(pkg.ADACONS_TUNE_SHORT_PATH, 2 if two else 0)
        probe.tune(pkg.ADACONS_TUNE_STATS_ONLY, stats_only)
        probe.profile_begin(2)
        probe.aggregate(G); probe.aggregate(G)
        assert (probe.profile_end()["coeff_ms"] == 0.0) == two
        probe.close()
    ost = o.OracleState(N, beta=0.9, flags=flags)
    for t in range(6):
        G = randG(N, d, dtype, sigma=2.0, seed=900 + t)
        if t == 2:
            G[N - 1].zero_()
        if t == 3:
            G[0, min(d - 1, 77)] = float("inf")
        a, b = short.aggregate(G).clone(), plain.aggregate(G).clone()
        ia, ib = short.coeffs(), plain.coeffs()
        assert torch.equal(a, b) or t == 3      # a non-finite input: NaN/Inf positions agree, compared below
        if t == 3:
            assert torch.equal(torch.isfinite(a), torch.isfinite(b)) and torch.equal(a[torch.isfinite(a)], b[torch.isfinite(b)])
        for key in ("gamma", "raw", "smoothed"):
            assert np.array_equal(ia[key], ib[key], equal_nan=True), (t, key)
        assert ia["numeric_flags"] == ib["numeric_flags"]
        if has_K:
            Ka, Kb = pkg.adacons_read_gram(short._st, N, None), pkg.adacons_read_gram(plain._st, N, None)
            assert np.array_equal(Ka, Kb, equal_nan=True)
        (ma, sa), (mb, sb) = short.export_state(), plain.export_state()
        assert np.array_equal(ma, mb) and sa == sb == t + 1
        # and against the oracle, like every other path
        state_was_zero = not ost.m.any()
        Gh = workloads.to_oracle_input(G)
        oout, oinfo = o.aggregate(Gh, ost, want_out=(t != 3))
        check_coefficients(ia, oinfo, ost.m, ost.flags, state_was_zero, ties_possible=(N == 1))
        if t != 3:
            check_out(a.cpu().numpy(), Gh, ia, oout, True)
    w1, w2 = torch.randn(d, device=DEV), None
    w2 = w1.clone()
    G = randG(N, d, dtype, sigma=2.0, seed=990)
    short.aggregate_apply(G, w1, lr=0.3)
    plain.aggregate_apply(G, w2, lr=0.3)
    assert torch.equal(w1, w2)
    # checkpoint taken on one path resumes on the other
    m, step = short.export_state()
    plain.import_state(m, step)
    G = randG(N, d, dtype, sigma=2.0, seed=991)
    assert torch.equal(short.aggregate(G), plain.aggregate(G))
    short.close(); plain.close()


def test_short_path_is_the_default_for_small_gradients_only(pkg):
    """Up to 32 MiB of gradients (N <= 8, aligned rows; bf16: 16 MiB for 2 < N <= 6, 8 MiB for N = 7, 8) take two
    launches, larger ones three; N > 8 up to 1 MiB, unless the Gram matrix takes more than one workgroup to
    reduce (44 < N <= 64): seen through the per-stage timing, which reports no time of its own for stage A2
    on the short path."""
    f32, bf16 = torch.float32, torch.bfloat16
    for N, d, dtype, short in [(4, 1 << 20, f32, True), (8, 1 << 20, f32, True), (8, (1 << 20) + 4, f32, False),
                               (4, 1001, f32, False), (2, 1 << 23, bf16, True), (2, (1 << 23) + 8, bf16, False),
                               (4, 1 << 21, bf16, True), (4, (1 << 21) + 8, bf16, False), (6, 1 << 20, bf16, True),
                               (8, 1 << 19, bf16, True), (8, (1 << 19) + 8, bf16, False), (7, 1 << 20, bf16, False),
                               (16, 1000, f32, True), (16, 16388, f32, False), (9, 1000, f32, True),
                               (32, 1000, f32, True), (32, 8192, f32, True), (32, 8196, f32, False),
                               (48, 1000, f32, False), (128, 1000, f32, True)]:
        agg = pkg.AdaCons(N, d)
        G = randG(N, d, dtype, seed=1)
        agg.aggregate(G)
        agg.profile_begin(20)
        for _ in range(20):
            agg.aggregate(G)
        prof = agg.profile_end()
        assert (prof["coeff_ms"] == 0.0) == short, (N, d, dtype, prof)
        agg.close()


@pytest.mark.parametrize("per_cu", [1, 2, 3])
def test_launch_shape_does_not_change_results_beyond_rounding(pkg, per_cu):
    N, d = 8, 2_000_000
    G = randG(N, d, seed=11)
    ost = o.OracleState(N)
    agg = pkg.AdaCons(N, d)
    agg.tune(pkg.ADACONS_TUNE_GRAM_BLOCKS_PER_CU, per_cu)
    agg.tune(pkg.ADACONS_TUNE_WSUM_BLOCKS_PER_CU, per_cu)
    both(pkg, G, agg, ost)
    agg.close()


# --------------------------------------------------------------------------- edge cases ----
@pytest.mark.parametrize("N,d", [(1, 1), (1, 513), (2, 1), (8, 3), (16, 1), (64, 2), (4, 255), (4, 1025)])
def test_tiny_and_ragged_shapes(pkg, N, d):
    G = randG(N, d, sigma=1.0, seed=N + d)
    agg = pkg.AdaCons(N, d, beta=0.7)
    ost = o.OracleState(N, beta=0.7)
    _, _, oinfo = both(pkg, G, agg, ost, ties_possible=(d == 1))
    assert oinfo["strict"]        # from a zero state the order of tied workers cannot matter
    # second and third step with the state carried: a one-column input ties every |a_i|, and the
    # comparison then covers what a tie leaves unique (and stage A3 with the weights the GPU chose)
    for t in (1, 2):
        both(pkg, randG(N, d, sigma=1.0, seed=N + d + 100 * t), agg, ost, ties_possible=(d == 1))
    m, step = agg.export_state()
    assert step == 3
    assert_gamma_close(m, ost.m)
    agg.close()


def shifted_rows(N, d, dtype, shift, seed=0):
    """An N x d contiguous view that starts `shift` elements into a fresh allocation."""
    flat = torch.empty(N * d + shift, device=DEV, dtype=dtype)
    G = flat[shift:].view(N, d)
    G.copy_(randG(N, d, dtype=dtype, seed=seed))   # a common signal plus noise: well-conditioned coefficients
    assert G.is_contiguous() and G.data_ptr() == flat.data_ptr() + shift * flat.element_size()
    return G


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("N", [4, 16])
def test_unaligned_base_and_odd_length(pkg, N, dtype):
    """G starting one element past a 16-byte boundary, odd d: 128-bit accesses from element-aligned
    addresses plus the kernels for the columns that no whole group covers."""
    d = 100_001
    G = shifted_rows(N, d, dtype, 1)
    assert G.data_ptr() % 16 != 0
    agg = pkg.AdaCons(N, d)
    both(pkg, G, agg, o.OracleState(N))
    outbuf = torch.empty(d + 1, device=DEV)
    agg2 = pkg.AdaCons(N, d)
    out2 = agg2.aggregate(G, out=outbuf[1:])
    assert rel_l2(out2.cpu().numpy(), agg.aggregate(G).cpu().numpy()) <= 1e-6
    agg.close(); agg2.close()


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("N,d,shift", [(1, 5, 1), (3, 2, 0), (5, 9, 3), (8, 70_003, 0), (8, 70_000, 2), (7, 262_150, 5),
                                       (8, 1_048_577, 0), (9, 7, 1), (16, 33, 0), (16, 70_001, 3), (24, 65_543, 0),
                                       (33, 20_002, 1), (48, 40_005, 0), (64, 131_079, 7), (64, 65_536, 1), (64, 6, 0)])
@pytest.mark.parametrize("stats_only", [0, 1])
def test_rows_off_16_byte_boundaries(pkg, N, d, shift, dtype, stats_only):
    """Every leftover count (d mod 4 for fp32, d mod 8 for bf16), shifted bases, d smaller than one
    group, all row-tile counts, with and without the statistics-only first pass, over two steps
    (momentum carried); then the fused descent step on the same input."""
    if stats_only and N <= 8:
        pytest.skip("statistics-only applies to N > 8")
    agg = pkg.AdaCons(N, d, beta=0.8)
    agg.tune(pkg.ADACONS_TUNE_STATS_ONLY, stats_only)
    ost = o.OracleState(N, beta=0.8)
    for t in range(2):
        G = shifted_rows(N, d, dtype, shift, seed=17 * N + t)
        both(pkg, G, agg, ost, ties_possible=(d == 1))
    if not stats_only:
        K = pkg.adacons_read_gram(agg._st, N, None)
        assert rel_l2(K, o.gram(workloads.to_oracle_input(G))) <= 3e-7
    # w <- w - lr * aggregate with an output that is itself off the 16-byte grid
    wbuf = torch.randn(d + 1, device=DEV)
    w = wbuf[1:]
    w0 = w.clone()
    state_was_zero = not ost.m.any()
    agg.aggregate_apply(G, w, lr=0.25)
    info = agg.coeffs()
    Gh = workloads.to_oracle_input(G)
    oout, oinfo = o.aggregate(Gh, ost)
    strict = check_coefficients(info, oinfo, ost.m, ost.flags, state_was_zero, ties_possible=(d == 1))
    assert_out_elementwise(w.cpu().numpy(), Gh, info["gamma"], base=w0.cpu().numpy(), lr=0.25)
    if strict:
        ref = w0.cpu().numpy().astype(np.float64) - 0.25 * oout
        assert rel_l2(w.cpu().numpy(), ref) <= 1e-5
    agg.close()


def test_d_smaller_than_d_max_and_state_reuse(pkg):
    N = 8
    agg = pkg.AdaCons(N, 1_000_000, beta=0.5)
    ost = o.OracleState(N, beta=0.5)
    for d in (1_000_000, 12, 400_004, 999_999):
        both(pkg, randG(N, d, seed=d % 13), agg, ost)
    agg.close()


def test_degenerate_inputs_match_oracle_flags(pkg):
    N, d = 4, 10_000
    agg = pkg.AdaCons(N, d, beta=0.5)
    ost = o.OracleState(N, beta=0.5)
    G = randG(N, d, seed=1)
    both(pkg, G, agg, ost)
    Gz = G.clone(); Gz[2] = 0
    _, info, _ = both(pkg, Gz, agg, ost)
    assert info["numeric_flags"] & pkg.ADACONS_NUM_ZERO_NORM and info["gamma"][2] == 0.0
    m_before, _ = agg.export_state()
    Gn = G.clone(); Gn[1, 77] = float("inf")
    out = agg.aggregate(Gn)
    info = agg.coeffs()
    oout, oinfo = o.aggregate(workloads.to_oracle_input(Gn), ost, want_out=False)
    assert info["numeric_flags"] == oinfo["numeric_flags"] == (pkg.ADACONS_NUM_NONFINITE | pkg.ADACONS_NUM_UNIFORM_FALLBACK)
    assert np.allclose(info["gamma"], 0.25)
    m_after, step = agg.export_state()
    assert np.array_equal(m_before, m_after) and step == 3 == ost.t
    _, info, _ = both(pkg, torch.zeros(N, d, device=DEV), agg, ost)
    assert info["numeric_flags"] & pkg.ADACONS_NUM_UNIFORM_FALLBACK
    g = torch.randn(d, device=DEV)
    agg2, ost2 = pkg.AdaCons(2, d), o.OracleState(2)
    _, info, _ = both(pkg, torch.stack([g, -g]).contiguous(), agg2, ost2)
    assert info["numeric_flags"] & pkg.ADACONS_NUM_UNIFORM_FALLBACK and np.allclose(info["gamma"], 0.5)
    agg.close(); agg2.close()


@pytest.mark.parametrize("N,dtype,stats_only", [(16, torch.float32, 0), (48, torch.float32, 0), (64, torch.float32, 0),
                                               (64, torch.bfloat16, 0), (32, torch.float32, 1), (64, torch.bfloat16, 1)])
def test_degenerate_inputs_many_workers(pkg, N, dtype, stats_only):
    """Zero rows, an infinity, a NaN and all-zero input through the matrix-core kernels (fp32
    instruction, split-bf16 products, bf16 instruction) and the statistics-only pass: same flags,
    same weights, momentum state untouched by a non-finite step."""
    d = 40_000
    agg = pkg.AdaCons(N, d, beta=0.5)
    agg.tune(pkg.ADACONS_TUNE_STATS_ONLY, stats_only)
    ost = o.OracleState(N, beta=0.5)
    G = randG(N, d, dtype=dtype, sigma=2.0, seed=N)
    both(pkg, G, agg, ost)
    Gz = G.clone(); Gz[N - 1] = 0; Gz[3] = 0
    _, info, _ = both(pkg, Gz, agg, ost)
    assert info["numeric_flags"] & pkg.ADACONS_NUM_ZERO_NORM and info["gamma"][3] == 0.0 and info["gamma"][N - 1] == 0.0
    m_before, _ = agg.export_state()
    for bad in (float("inf"), float("-inf"), float("nan")):
        Gn = G.clone(); Gn[N // 2, 12_345] = bad
        agg.aggregate(Gn)
        info = agg.coeffs()
        _, oinfo = o.aggregate(workloads.to_oracle_input(Gn), ost, want_out=False)
        assert info["numeric_flags"] == oinfo["numeric_flags"] == (pkg.ADACONS_NUM_NONFINITE | pkg.ADACONS_NUM_UNIFORM_FALLBACK)
        assert np.allclose(info["gamma"], 1.0 / N)
    m_after, step = agg.export_state()
    assert np.array_equal(m_before, m_after) and step == 5 == ost.t
    _, info, _ = both(pkg, torch.zeros(N, d, device=DEV, dtype=dtype), agg, ost)
    assert info["numeric_flags"] & pkg.ADACONS_NUM_UNIFORM_FALLBACK
    both(pkg, G, agg, ost)          # and a regular step afterwards
    agg.close()


def test_checkpoint_resume_and_reset(pkg):
    N, d = 8, 200_000
    a = pkg.AdaCons(N, d, beta=0.9)
    Gs = [randG(N, d, sigma=2.0, seed=70 + t) for t in range(6)]
    for G in Gs[:3]:
        a.aggregate(G)
    m, step = a.export_state()
    b = pkg.AdaCons(N, d, beta=0.9)
    b.import_state(m, step)
    for G in Gs[3:]:
        oa, ob = a.aggregate(G), b.aggregate(G)
        assert torch.equal(oa, ob)
        assert np.array_equal(a.coeffs()["gamma"], b.coeffs()["gamma"])
    a.reset()
    m0, s0 = a.export_state()
    assert not m0.any() and s0 == 0
    c = pkg.AdaCons(N, d, beta=0.9)
    assert torch.equal(a.aggregate(Gs[0]), c.aggregate(Gs[0]))
    a.close(); b.close(); c.close()


def test_error_codes_on_the_gpu(pkg):
    N, d = 4, 1000
    agg = pkg.AdaCons(N, d)
    G = randG(N, d)
    out = torch.empty(d, device=DEV)
    with pytest.raises(pkg.AdaConsError) as e:
        pkg.adacons_aggregate(randG(N, d + 1), agg._st, torch.empty(d + 1, device=DEV))
    assert e.value.status == 1
    with pytest.raises(pkg.AdaConsError) as e:
        pkg.adacons_aggregate(randG(N + 1, d), agg._st, out)
    assert e.value.status == 1
    with pytest.raises(pkg.AdaConsError) as e:                     # out aliases the last row of G
        pkg.adacons_aggregate(G, agg._st, G[N - 1])
    assert e.value.status == 1
    agg.aggregate(G, out=out)                                       # still usable afterwards
    assert torch.isfinite(out).all()
    agg.close()


def test_tuning_values_are_validated_and_restored(pkg):
    """adacons_tune rejects values outside a key's documented range with ADACONS_EINVAL and leaves the
    setting alone; a negative value restores the default (same bits as a fresh state)."""
    N, d = 32, 4096
    G = randG(N, d, seed=21)
    agg, fresh = pkg.AdaCons(N, d), pkg.AdaCons(N, d)
    for key, bad in [(pkg.ADACONS_TUNE_GRAM_BLOCKS_PER_CU, 9), (pkg.ADACONS_TUNE_WSUM_BLOCKS_PER_CU, 9),
                     (pkg.ADACONS_TUNE_GRAM_PRODUCTS, 3), (pkg.ADACONS_TUNE_SHORT_PATH, 3),
                     (pkg.ADACONS_TUNE_WSUM_ROW_SLICES, 3), (pkg.ADACONS_TUNE_WSUM_PARK_KB, 4),
                     (pkg.ADACONS_TUNE_WSUM_PARK_KB, 145), (8, 0), (-1, 0)]:
        with pytest.raises(pkg.AdaConsError) as e:
            agg.tune(key, bad)
        assert e.value.status == 1, (key, bad)        # ADACONS_EINVAL
    assert torch.equal(agg.aggregate(G), fresh.aggregate(G))      # nothing was changed by the rejected calls
    agg.tune(pkg.ADACONS_TUNE_WSUM_ROW_SLICES, 0)
    agg.tune(pkg.ADACONS_TUNE_SHORT_PATH, 0)
    agg.tune(pkg.ADACONS_TUNE_WSUM_ROW_SLICES, -1)
    agg.tune(pkg.ADACONS_TUNE_SHORT_PATH, -1)
    assert torch.equal(agg.aggregate(G), fresh.aggregate(G))      # defaults restored
    agg.close(); fresh.close()


def test_non_default_stream(pkg):
    N, d = 8, 500_000
    G = randG(N, d, seed=21)
    ref = pkg.AdaCons(N, d)
    want = ref.aggregate(G).clone()
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    agg = pkg.AdaCons(N, d, stream=s)
    with torch.cuda.stream(s):
        out = agg.aggregate(G)
        gam = agg.coeffs()["gamma"]
    s.synchronize()
    assert torch.equal(out, want) and np.array_equal(gam, ref.coeffs()["gamma"])
    agg.close(); ref.close()


# --------------------------------------------------------------- fused descent step (Eq. 4) ----
@pytest.mark.parametrize("N,d,dtype", [(8, 1_000_004, torch.float32), (4, 100_003, torch.float32),
                                       (16, 200_000, torch.float32), (64, 50_000, torch.float32),
                                       (8, 400_008, torch.bfloat16)])
def test_aggregate_apply_is_the_descent_step(pkg, N, d, dtype):
    """w <- w - lr * psi (Eq. 4 with Eq. 12) in one pass, against w - lr * (oracle aggregate) in float64,
    over several steps with the momentum state carried along."""
    lr = 0.05
    agg = pkg.AdaCons(N, d, beta=0.9)
    ost = o.OracleState(N, beta=0.9)
    w = torch.randn(d, device=DEV)
    w_ref = w.cpu().numpy().astype(np.float64)
    for t in range(3):
        G = randG(N, d, dtype, sigma=2.0, seed=500 + t)
        w_before = w.cpu().numpy()
        agg.aggregate_apply(G, w, lr)
        info = agg.coeffs()
        Gh = workloads.to_oracle_input(G)
        psi, oinfo = o.aggregate(Gh, ost)
        w_ref = w_ref - lr * psi
        assert_gamma_close(info["gamma"], oinfo["gamma"])
        assert rel_l2(w.cpu().numpy(), w_ref) <= 1e-6
        # the step itself, element by element: w_before - lr * (weighted sum of the applied weights)
        assert_out_elementwise(w.cpu().numpy(), Gh, info["gamma"], base=w_before, lr=lr)
    agg.close()


def test_aggregate_apply_rejects_bad_arguments(pkg):
    N, d = 4, 1000
    agg = pkg.AdaCons(N, d)
    G = randG(N, d)
    with pytest.raises(pkg.AdaConsError):
        agg.aggregate_apply(G, G[0], 0.1)                      # w overlaps G
    with pytest.raises(pkg.AdaConsError):
        agg.aggregate_apply(G, torch.zeros(d, device=DEV), float("nan"))
    agg.close()


# --------------------------------------------------------- statistics-only first pass ----
@pytest.mark.parametrize("N,d", [(9, 70_000), (16, 200_000), (16, 16), (17, 50_008), (32, 65_536 + 24), (33, 10_000),
                                 (48, 30_000), (63, 10_008), (64, 131_072 + 24), (64, 8)])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_statistics_only_first_pass_matches_oracle(pkg, N, d, dtype):
    """ADACONS_TUNE_STATS_ONLY: A1 delivers only diag K and the row sums of K (what Eq. 7 consumes);
    coefficients, momentum state and output must match the oracle over several steps, and K is
    reported as not available."""
    agg = pkg.AdaCons(N, d, beta=0.9)
    agg.tune(pkg.ADACONS_TUNE_STATS_ONLY, 1)
    ost = o.OracleState(N, beta=0.9)
    for t in range(3):
        G = randG(N, d, dtype=dtype, sigma=2.0, seed=1000 * N + t)
        both(pkg, G, agg, ost)
    with pytest.raises(pkg.AdaConsError) as e:
        pkg.adacons_read_gram(agg._st, N, None)
    assert e.value.status == 1        # ADACONS_EINVAL
    m, step = agg.export_state()
    assert step == 3 and np.allclose(m, ost.m, rtol=1e-6, atol=0)
    agg.gram(G)                       # a Gram call makes K available again
    agg.close()


def test_statistics_only_is_ignored_where_it_does_not_apply(pkg):
    """N <= 8 keeps the Gram kernel (K stays available)."""
    N, d = 8, 100_000
    G = randG(N, d, seed=2)
    agg = pkg.AdaCons(N, d)
    agg.tune(pkg.ADACONS_TUNE_STATS_ONLY, 1)
    both(pkg, G, agg, o.OracleState(N))
    K = pkg.adacons_read_gram(agg._st, N, None)
    assert rel_l2(K, o.gram(workloads.to_oracle_input(G))) <= 3e-7
    agg.close()


def test_statistics_only_degenerate_rows(pkg):
    """Zero rows and identical rows through the statistics-only pass: same flags and weights."""
    N, d = 16, 40_000
    G = randG(N, d, sigma=1.0, seed=5)
    G[3].zero_()
    G[7] = G[6]
    agg = pkg.AdaCons(N, d)
    agg.tune(pkg.ADACONS_TUNE_STATS_ONLY, 1)
    ost = o.OracleState(N)
    out = agg.aggregate(G)
    info = agg.coeffs()
    Gh = workloads.to_oracle_input(G)
    oout, oinfo = o.aggregate(Gh, ost)
    assert info["numeric_flags"] == oinfo["numeric_flags"] != 0
    assert check_coefficients(info, oinfo, ost.m, ost.flags, True)
    check_out(out.cpu().numpy(), Gh, info, oout, True)
    agg.close()


# ------------------------------------------------------------- parked output (stage A3) ----
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("N,d,park_kb", [(3, 3_000_003, 8), (8, 3_000_000, 24), (8, 4_194_304, 40),
                                         (16, 2_000_004, 16), (4, 2_500_000, 128), (40, 1_500_008, 48),
                                         (128, 600_000, 144), (8, 1000, 128), (5, 2_100_000, 32)])
def test_parked_output_matches_oracle_and_plain_kernel(pkg, N, d, park_kb, dtype):
    """ADACONS_TUNE_WSUM_PARK_KB: whole output tiles parked in LDS and written in bursts -- several
    bursts per workgroup, a partial last tile, a ragged d; the
    output must equal the plain kernel's bit for bit (same sums, only the time of the store differs),
    and the fused descent step must agree with it too."""
    G = randG(N, d, dtype=dtype, sigma=2.0, seed=5 * N + park_kb)
    ref_agg = pkg.AdaCons(N, d)
    ref_agg.tune(pkg.ADACONS_TUNE_WSUM_PARK_KB, 0)
    ref = ref_agg.aggregate(G).clone()
    agg = pkg.AdaCons(N, d)
    agg.tune(pkg.ADACONS_TUNE_WSUM_PARK_KB, park_kb)
    out, info, oinfo = both(pkg, G, agg, o.OracleState(N))
    assert torch.equal(out, ref)
    w = torch.randn(d, device=DEV)
    w_ref = w.clone()
    agg.aggregate_apply(G, w, lr=0.5)
    ref_agg.aggregate_apply(G, w_ref, lr=0.5)
    assert torch.equal(w, w_ref)
    agg.close(); ref_agg.close()


@pytest.mark.parametrize("N,d", [(12, (1 << 24) + 4100), (5, 70_000_004)])
def test_parked_output_is_the_default_for_long_fp32_streams(pkg, N, d):
    """fp32, d >= 2^24, and N >= 12 or 1.25 GiB of gradients through the run-time-N kernel: the default
    second pass parks its output; bit-identical to the plain kernel (ADACONS_TUNE_WSUM_PARK_KB = 0).
    Values other than 0, 1, 8..144 are rejected."""
    G = randG(N, d, sigma=2.0, seed=3)
    plain = pkg.AdaCons(N, d)
    plain.tune(pkg.ADACONS_TUNE_WSUM_PARK_KB, 0)
    dflt = pkg.AdaCons(N, d)
    a, b = plain.aggregate(G).clone(), dflt.aggregate(G).clone()
    assert torch.equal(a, b)
    for bad in (2, 7, 145):
        with pytest.raises(pkg.AdaConsError) as e:
            dflt.tune(pkg.ADACONS_TUNE_WSUM_PARK_KB, bad)
        assert e.value.status == 1
    plain.close(); dflt.close()


# ------------------------------------------------------------------ more than 64 workers ----
@pytest.mark.parametrize("N,d", [(65, 1_000), (65, 40_003), (80, 20_000), (96, 65_536 + 24), (97, 10_001), (112, 30_000),
                                 (127, 9_999), (128, 131_072 + 8), (128, 5), (128, 1), (128, 4_000_004)])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_more_than_64_workers(pkg, N, d, dtype):
    """64 < N <= 128 (the paper's linear-regression runs go up to 128 workers): stage A1 is the
    statistics pass (norms and dot products with the summed gradient, Alg. 1 steps 1-2), K is not
    formed; coefficients, momentum state and output over three steps against the oracle."""
    agg = pkg.AdaCons(N, d, beta=0.9)
    ost = o.OracleState(N, beta=0.9)
    for t in range(3):
        G = randG(N, d, dtype=dtype, sigma=2.0, seed=77 * N + t)
        _, _, oinfo = both(pkg, G, agg, ost, ties_possible=(d == 1))
        assert oinfo["strict"] or d == 1
    with pytest.raises(pkg.AdaConsError) as e:
        pkg.adacons_read_gram(agg._st, N, None)
    assert e.value.status == 1        # ADACONS_EINVAL
    with pytest.raises(pkg.AdaConsError) as e:
        agg.gram(G)
    assert e.value.status == 2        # ADACONS_EUNSUPPORTED
    m, step = agg.export_state()
    assert step == 3 and np.allclose(m, ost.m, rtol=1e-6, atol=0)
    # stage A3 alone with given weights, and the fused descent step
    gamma = np.linspace(-0.5, 1.5, N)
    out = agg.weighted_sum(G, gamma)
    ref = o.weighted_sum(workloads.to_oracle_input(G), gamma.astype(np.float32).astype(np.float64))
    assert rel_l2(out.cpu().numpy(), ref) <= 1e-5
    w = torch.randn(d, device=DEV)
    w0 = w.clone()
    agg.aggregate_apply(G, w, lr=0.5)
    info = agg.coeffs()
    Gh = workloads.to_oracle_input(G)
    oout, oinfo = o.aggregate(Gh, ost)
    strict = check_coefficients(info, oinfo, ost.m, ost.flags, False, ties_possible=(d == 1))
    assert_out_elementwise(w.cpu().numpy(), Gh, info["gamma"], base=w0.cpu().numpy(), lr=0.5)
    if strict:
        assert rel_l2(w.cpu().numpy(), w0.cpu().numpy().astype(np.float64) - 0.5 * oout) <= 1e-5
    agg.close()


@pytest.mark.parametrize("flags", [0, 1, 2, 3, 7, 11, 15])
def test_more_than_64_workers_ablation_flags(pkg, flags):
    N, d = 100, 20_000
    agg = pkg.AdaCons(N, d, beta=0.9, flags=flags)
    ost = o.OracleState(N, beta=0.9, flags=flags)
    for t in range(3):
        G = randG(N, d, sigma=2.0, seed=300 + t)
        if flags & 4:
            G = G[torch.roll(torch.arange(N), t).to(DEV)].contiguous()
        both(pkg, G, agg, ost)
    m, _ = agg.export_state()
    assert np.allclose(m, ost.m, rtol=1e-6, atol=1e-12)
    agg.close()


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_more_than_64_workers_degenerate_inputs(pkg, dtype):
    N, d = 128, 30_000
    agg = pkg.AdaCons(N, d, beta=0.5)
    ost = o.OracleState(N, beta=0.5)
    G = randG(N, d, dtype=dtype, sigma=2.0, seed=9)
    both(pkg, G, agg, ost)
    Gz = G.clone(); Gz[N - 1] = 0; Gz[70] = 0; Gz[100] = Gz[99]
    _, info, _ = both(pkg, Gz, agg, ost)
    assert info["numeric_flags"] & pkg.ADACONS_NUM_ZERO_NORM and info["gamma"][70] == 0.0 and info["gamma"][N - 1] == 0.0
    m_before, _ = agg.export_state()
    for bad in (float("inf"), float("nan")):
        Gn = G.clone(); Gn[90, 12_345] = bad
        agg.aggregate(Gn)
        info = agg.coeffs()
        _, oinfo = o.aggregate(workloads.to_oracle_input(Gn), ost, want_out=False)
        assert info["numeric_flags"] == oinfo["numeric_flags"] == (pkg.ADACONS_NUM_NONFINITE | pkg.ADACONS_NUM_UNIFORM_FALLBACK)
        assert np.allclose(info["gamma"], 1.0 / N)
    m_after, step = agg.export_state()
    assert np.array_equal(m_before, m_after) and step == 4 == ost.t
    _, info, _ = both(pkg, torch.zeros(N, d, device=DEV, dtype=dtype), agg, ost)
    assert info["numeric_flags"] & pkg.ADACONS_NUM_UNIFORM_FALLBACK
    agg.close()


# ------------------------------------------------------------------------- graph capture ----
@pytest.mark.parametrize("N,d,park_kb", [(8, 1_000_004, 1), (16, 600_000, 96), (4, 65_536, 1), (32, 8192, 1), (128, 1000, 1)])
def test_aggregate_can_be_captured_in_a_hip_graph(pkg, N, d, park_kb):
    """adacons_aggregate enqueues kernels only (no allocation, no synchronisation, no memset
    node), so a caller may capture it; every replay advances the momentum state like an eager
    call.  Replays are interleaved with eager work and checked one by one against the oracle.
    Second case: the matrix-core Gram pass and the second pass with its output parked in LDS; third: the
    two-launch short path (its parity flip happens on the device); fourth and fifth: many workers with
    short gradients (second pass by row slices; statistics-only first pass for N > 64)."""
    agg = pkg.AdaCons(N, d, beta=0.9)
    agg.tune(pkg.ADACONS_TUNE_WSUM_PARK_KB, park_kb)
    ost = o.OracleState(N, beta=0.9)
    G = randG(N, d, sigma=2.0, seed=77)
    out = torch.empty(d, device=DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        agg.aggregate(G, out=out, stream=side)          # warm-up call outside the capture
    side.synchronize()
    o.aggregate(workloads.to_oracle_input(G), ost, want_out=False)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        agg.aggregate(G, out=out, stream=torch.cuda.current_stream())
    for rep in range(4):
        G.copy_(randG(N, d, sigma=2.0, seed=80 + rep))   # eager work between replays: new input in place
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        info = agg.coeffs()
        Gh = workloads.to_oracle_input(G)
        ref_out, ref = o.aggregate(Gh, ost)
        assert check_coefficients(info, ref, ost.m, ost.flags, False)
        check_out(out.cpu().numpy(), Gh, info, ref_out, True)
    _, step = agg.export_state()
    assert step == 5
    agg.close()


# ------------------------------------------------------------------- randomized sweep ----
def test_randomized_shapes_flags_and_tunings(pkg):
    """A seeded sweep over what the other tests fix one at a time: worker count (all kernel families and
    their boundaries), length, dtype, ablation flags, base alignment, and every tuning key that selects a
    kernel (statistics-only, row slices, short path, Gram products), three steps with the state carried,
    the last one sometimes as the fused descent step.  Every step is checked like any other."""
    rng = np.random.default_rng(20241103)
    Ns = [1, 2, 3, 4, 5, 7, 8, 9, 12, 15, 16, 17, 24, 31, 32, 33, 44, 45, 48, 63, 64, 65, 96, 127, 128]
    for case in range(120):
        N = int(rng.choice(Ns))
        d = int(np.exp(rng.uniform(np.log(600), np.log(300_000 if N <= 32 else 50_000))))
        dtype = torch.float32 if rng.random() < 0.5 else torch.bfloat16
        flags = int(rng.choice([0, 1, 2, 3, 3, 3, 7, 11, 15]))
        shift = int(rng.integers(1, 8)) if rng.random() < 0.3 else 0
        tunes = [(pkg.ADACONS_TUNE_STATS_ONLY, int(rng.random() < 0.3)), (pkg.ADACONS_TUNE_WSUM_ROW_SLICES, int(rng.choice([0, 1, 1, 2]))),
                 (pkg.ADACONS_TUNE_SHORT_PATH, int(rng.choice([0, 1, 1, 2]))), (pkg.ADACONS_TUNE_GRAM_PRODUCTS, int(rng.choice([0, 1, 2])))]
        apply_last = rng.random() < 0.5
        what = (case, N, d, dtype, flags, shift, tunes, apply_last)
        agg = pkg.AdaCons(N, d, beta=0.9, flags=flags)
        for key, value in tunes:
            agg.tune(key, value)
        ost = o.OracleState(N, beta=0.9, flags=flags)
        for t in range(3):
            G = shifted_rows(N, d, dtype, shift, seed=1000 * case + t)
            if apply_last and t == 2:
                w = torch.randn(d, device=DEV)
                w0 = w.cpu().numpy()
                state_was_zero = not ost.m.any()
                agg.aggregate_apply(G, w, lr=0.125)
                info = agg.coeffs()
                Gh = workloads.to_oracle_input(G)
                _, oinfo = o.aggregate(Gh, ost, want_out=False)
                assert check_coefficients(info, oinfo, ost.m, ost.flags, state_was_zero), what
                assert_out_elementwise(w.cpu().numpy(), Gh, info["gamma"], base=w0, lr=0.125)
            else:
                _, _, oinfo = both(pkg, G, agg, ost)
                assert oinfo["strict"], what
        agg.close()
