"""Pins of the float64 oracle to what the paper and the mathematics fix.

The paper prints no numeric worked example of the aggregator, so the oracle is
pinned by library routines, closed forms, brute force and invariants instead:
each test names the step it pins and the passage it follows.
"""
import numpy as np
import pytest
import torch

from oracle import adacons_oracle as o

RNG = np.random.default_rng(20241103)


def _randG(N, d, sigma=1.0, rng=RNG):
    s = rng.standard_normal(d)
    return (s[None, :] + sigma * rng.standard_normal((N, d))).astype(np.float32)


def _to_bf16_bits(x32: np.ndarray) -> np.ndarray:
    t = torch.from_numpy(np.ascontiguousarray(x32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def _bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def _state(N, beta=0.99, mom=True, norm=True):
    flags = (o.FLAG_MOMENTUM if mom else 0) | (o.FLAG_NORMALIZE if norm else 0)
    return o.OracleState(N, beta=beta, flags=flags)


# ---------------------------------------------------------------- O1 / O2 ----
@pytest.mark.parametrize("N,d", [(1, 1), (2, 7), (5, 65535), (8, 65536), (3, 65537),
                                 (17, 3 * 65536 + 11), (64, 4099)])
def test_gram_equals_library_matmul_f32(N, d):
    """O1: K = G G^T (Eq. 7 third line) reduces to a float64 library matmul."""
    G = _randG(N, d)
    K = o.gram(G)
    G64 = G.astype(np.float64)
    ref = G64 @ G64.T
    assert np.allclose(K, ref, rtol=1e-12, atol=1e-9 * d ** 0.5)
    assert np.array_equal(K, K.T)
    assert (np.diag(K) >= 0).all()
    assert np.linalg.eigvalsh(K).min() >= -1e-9 * np.trace(K)


@pytest.mark.parametrize("N,d", [(2, 5), (8, 65536 + 123), (16, 70001)])
def test_gram_equals_library_matmul_bf16(N, d):
    """O1 with bf16 storage: widening is exact, products taken in float64."""
    bits = _to_bf16_bits(_randG(N, d, sigma=2.0))
    K = o.gram(bits)
    G64 = _bf16_bits_to_f64(bits)
    assert np.allclose(K, G64 @ G64.T, rtol=1e-12, atol=1e-9 * d ** 0.5)


def test_gram_is_not_transposed_or_offset():
    """A wrong row stride or a transposed operand shows on a matrix with distinct rows."""
    N, d = 3, 5
    G = np.arange(1, N * d + 1, dtype=np.float32).reshape(N, d)
    K = o.gram(G)
    expect = np.array([[55, 130, 205], [130, 330, 530], [205, 530, 855]], dtype=np.float64)
    assert np.array_equal(K, expect)


def test_row_sums_are_dot_with_sum_of_gradients():
    """O2/O3: r_i = <g_i, sum_j g_j>, so a_i = <g_i, gbar>/||g_i|| (Eq. 7, second line)."""
    N, d = 6, 2000
    G = _randG(N, d)
    st = _state(N, mom=False, norm=False)
    _, info = o.aggregate(G, st, want_out=False)
    G64 = G.astype(np.float64)
    gbar = G64.mean(0)
    a = (G64 @ gbar) / np.linalg.norm(G64, axis=1)
    assert np.allclose(info["raw"], a, rtol=1e-12)


# --------------------------------------------------------------------- O3 ----
def test_first_order_coefficient_is_subspace_gradient_on_quadratic():
    """O3 by brute force: central differences of h(alpha) = f(w + P alpha) at 0
    (Eq. 5-6) on a quadratic f whose gradient at w is the mean gradient (Sec. 3.2),
    with column-normalised P, equal <g_i, gbar>/||g_i|| (Eq. 7)."""
    N, d = 4, 7
    G = _randG(N, d, sigma=0.8)
    G64 = G.astype(np.float64)
    gbar = G64.mean(0)
    B = RNG.standard_normal((d, d))
    A = B @ B.T + np.eye(d)
    w = RNG.standard_normal(d)

    def f(x):
        return 0.5 * (x - w) @ A @ (x - w) + gbar @ (x - w)

    P = (G64 / np.linalg.norm(G64, axis=1, keepdims=True)).T      # d x N
    eps = 1e-4
    grad = np.array([(f(w + eps * P[:, i]) - f(w - eps * P[:, i])) / (2 * eps) for i in range(N)])
    _, info = o.aggregate(G, _state(N, mom=False, norm=False), want_out=False)
    assert np.allclose(info["raw"], grad, rtol=1e-7, atol=1e-9)
    assert (np.sign(info["raw"]) == np.sign(grad)).all()


# --------------------------------------------------------------------- O6 ----
def test_unnormalised_update_is_preconditioned_mean_gradient():
    """O6/O7 with lambda = 1 and no momentum: sum_i c_i g_i equals the explicit d x d
    preconditioner (sum_i g_i g_i^T / ||g_i||^2) applied to gbar (Eq. 9); it is PSD,
    hence a descent direction (Sec. 3.3)."""
    N, d = 5, 9
    G = _randG(N, d, sigma=1.5)
    G64 = G.astype(np.float64)
    gbar = G64.mean(0)
    M = sum(np.outer(g, g) / (g @ g) for g in G64)
    out, info = o.aggregate(G, _state(N, mom=False, norm=False))
    assert np.allclose(out, M @ gbar, rtol=1e-12, atol=1e-14)
    assert out @ gbar >= 0
    assert np.isclose(out @ gbar, sum((g @ gbar) ** 2 / (g @ g) for g in G64), rtol=1e-12)


def test_unnormalised_identical_gradients_give_the_sum():
    """lambda = 1 (Eq. 8): identical gradients give c_i = 1, i.e. the plain sum."""
    g = RNG.standard_normal(50).astype(np.float32)
    G = np.tile(g, (4, 1))
    out, info = o.aggregate(G, _state(4, mom=False, norm=False))
    assert np.allclose(info["gamma"], 1.0, rtol=1e-14)
    assert np.allclose(out, 4 * g.astype(np.float64), rtol=1e-14)


# ---------------------------------------------------------------- O4 / O5 ----
def test_sorted_ema_matches_closed_form_of_recurrence():
    """O4-O5 (Eq. 11): from zero state m_T = (1-beta) sum_tau beta^(T-tau) sort(a_tau), and
    worker i receives the entry at its own rank."""
    N, d, T, beta = 7, 300, 12, 0.9
    st = _state(N, beta=beta)
    raws = []
    for t in range(T):
        G = _randG(N, d, sigma=2.0)
        _, info = o.aggregate(G, st, want_out=False)
        raws.append(info["raw"].copy())
        m_closed = sum((1 - beta) * beta ** (t - tau) * np.sort(raws[tau]) for tau in range(t + 1))
        assert np.allclose(st.m, m_closed, rtol=1e-12, atol=1e-15)
        rank = np.argsort(np.argsort(raws[t], kind="stable"), kind="stable")
        assert np.allclose(info["smoothed"], m_closed[rank], rtol=1e-12, atol=1e-15)
        assert (np.diff(st.m) >= 0).all()          # an EMA of sorted vectors stays sorted
    assert st.t == T


def test_sorted_ema_ascending_with_stable_ties():
    """Sort direction/ties: ascending, ties to the lower worker index first."""
    K = np.diag([4.0, 1.0, 1.0, 9.0])
    # rows orthogonal: a_i = sqrt(q_i)/N  -> a = [0.5, 0.25, 0.25, 0.75]
    st = _state(4, beta=0.5)
    info = o.coefficients(K, st)
    assert np.allclose(info["raw"], [0.5, 0.25, 0.25, 0.75])
    assert np.allclose(st.m, 0.5 * np.array([0.25, 0.25, 0.5, 0.75]))
    # second call, different order: worker 3 now smallest
    K2 = np.diag([4.0, 1.0, 16.0, 0.25])
    info2 = o.coefficients(K2, st)         # a = [0.5, 0.25, 1.0, 0.125]
    m2 = 0.5 * 0.5 * np.array([0.25, 0.25, 0.5, 0.75]) + 0.5 * np.array([0.125, 0.25, 0.5, 1.0])
    assert np.allclose(st.m, m2)
    assert np.allclose(info2["smoothed"], m2[[2, 1, 3, 0]])
    # third call: workers 0 and 3 tie at the bottom; the state entries at ranks 0 and 1 now
    # differ, so the tie rule is visible: the lower index takes the lower rank
    K3 = np.diag([1.0, 4.0, 16.0, 1.0])    # a = [0.25, 0.5, 1.0, 0.25]
    info3 = o.coefficients(K3, st)
    m3 = 0.5 * m2 + 0.5 * np.array([0.25, 0.25, 0.5, 1.0])
    assert m3[0] != m3[1]
    assert np.allclose(st.m, m3)
    assert np.allclose(info3["smoothed"], m3[[0, 2, 3, 1]])


@pytest.mark.parametrize("beta", [0.0, 0.5, 0.99])
def test_first_step_from_zero_state_equals_momentum_off(beta):
    """From m = 0 the first EMA step is (1-beta) sort(a): a common factor the normalisation removes."""
    N, d = 9, 500
    G = _randG(N, d, sigma=3.0)
    out_m, info_m = o.aggregate(G, _state(N, beta=beta, mom=True))
    out_0, info_0 = o.aggregate(G, _state(N, beta=beta, mom=False))
    assert np.allclose(info_m["gamma"], info_0["gamma"], rtol=1e-12)
    assert np.allclose(out_m, out_0, rtol=1e-10, atol=1e-13)


def test_permutation_of_workers_with_persisting_state():
    """Sec. 3.4: the coefficient is decoupled from the worker index.  Permuting the rows at
    every step (state persisting) permutes gamma and leaves the aggregate unchanged."""
    N, d, T = 8, 400, 10
    st_a, st_b = _state(N, beta=0.9), _state(N, beta=0.9)
    for t in range(T):
        G = _randG(N, d, sigma=2.0)
        perm = RNG.permutation(N)
        out_a, info_a = o.aggregate(G, st_a)
        out_b, info_b = o.aggregate(G[perm], st_b)
        assert np.allclose(info_b["gamma"], info_a["gamma"][perm], rtol=1e-11)
        assert np.allclose(out_b, out_a, rtol=1e-9, atol=1e-12)
        assert np.allclose(st_a.m, st_b.m, rtol=1e-13)


def test_index_coupled_ema_is_the_plain_recurrence_and_depends_on_worker_order():
    """Variant INDEX_EMA (Eq. 10): m_T[i] = (1-beta) sum_tau beta^(T-tau) a_tau[i] per worker index.
    Unlike the sorted EMA of Eq. 11 it is not invariant to re-ordering the workers between steps
    (the reason Sec. 3.3 gives for sorting), and it coincides with Eq. 11 while the coefficients
    keep their ascending order."""
    N, d, T, beta = 6, 300, 8, 0.8
    flags = o.FLAG_DEFAULT | o.FLAG_INDEX_EMA
    st = o.OracleState(N, beta=beta, flags=flags)
    st_perm = o.OracleState(N, beta=beta, flags=flags)
    raws, moved = [], 0.0
    for t in range(T):
        G = _randG(N, d, sigma=2.0)
        out, info = o.aggregate(G, st)
        raws.append(info["raw"].copy())
        m_closed = sum((1 - beta) * beta ** (t - tau) * raws[tau] for tau in range(t + 1))
        assert np.allclose(st.m, m_closed, rtol=1e-12, atol=1e-15)
        assert np.allclose(info["smoothed"], m_closed, rtol=1e-12, atol=1e-15)
        assert abs(info["gamma"].sum() - 1.0) < 1e-12
        perm = np.roll(np.arange(N), t + 1)
        out_p, _ = o.aggregate(G[perm], st_perm)
        if t > 0:
            moved = max(moved, np.linalg.norm(out_p - out) / np.linalg.norm(out))
    assert moved > 1e-3
    # orthogonal rows with norms growing with the index (a_i = ||g_i|| / N ascending at every
    # step): the sorted and the index-coupled EMA then agree
    st_i = o.OracleState(N, beta=beta, flags=flags)
    st_s = o.OracleState(N, beta=beta, flags=o.FLAG_DEFAULT)
    for t in range(4):
        K = np.diag(np.sort(RNG.uniform(0.5, 9.0, N)))
        a = o.coefficients(K, st_i)
        b = o.coefficients(K, st_s)
        assert (np.diff(a["raw"]) > 0).all()
        assert np.allclose(a["gamma"], b["gamma"], rtol=1e-13)
        assert np.allclose(st_i.m, st_s.m, rtol=1e-13)


def test_lambda_as_printed_in_eq13_normalises_the_subspace_coefficients():
    """Variant LAMBDA_EQ13: lambda = 1 / sum_k a~_k.  Then the coefficients on the column-normalised
    subspace matrix, gamma_i ||g_i||, sum to one; the weights are the default ones times
    sum(c) / sum(a~); identical gradients give the unit vector g / ||g|| (not the mean: why the
    default reading normalises the weights instead)."""
    N, d = 7, 500
    G = _randG(N, d, sigma=1.5)
    flags = o.FLAG_DEFAULT | o.FLAG_LAMBDA_EQ13
    out_l, lit = o.aggregate(G, o.OracleState(N, beta=0.9, flags=flags))
    out_d, dflt = o.aggregate(G, o.OracleState(N, beta=0.9, flags=o.FLAG_DEFAULT))
    norms = np.linalg.norm(G.astype(np.float64), axis=1)
    assert abs((lit["gamma"] * norms).sum() - 1.0) < 1e-12
    c = dflt["smoothed"] / norms
    assert np.allclose(lit["gamma"], dflt["gamma"] * c.sum() / dflt["smoothed"].sum(), rtol=1e-12)
    assert np.allclose(lit["raw"], dflt["raw"], rtol=1e-15)
    g = RNG.standard_normal(d).astype(np.float32)
    out, info = o.aggregate(np.tile(g, (4, 1)), o.OracleState(4, flags=flags))
    assert np.allclose(out, g.astype(np.float64) / np.linalg.norm(g.astype(np.float64)), rtol=1e-12)
    # without NORMALIZE the switch has nothing to act on
    _, a = o.aggregate(G, o.OracleState(N, flags=o.FLAG_MOMENTUM | o.FLAG_LAMBDA_EQ13))
    _, b = o.aggregate(G, o.OracleState(N, flags=o.FLAG_MOMENTUM))
    assert np.array_equal(a["gamma"], b["gamma"])


def test_constant_input_gives_constant_weights_over_time():
    N, d = 6, 256
    G = _randG(N, d, sigma=1.0)
    st = _state(N, beta=0.8)
    g0 = None
    for _ in range(6):
        _, info = o.aggregate(G, st, want_out=False)
        g0 = info["gamma"] if g0 is None else g0
        assert np.allclose(info["gamma"], g0, rtol=1e-12)


# --------------------------------------------------------------------- O7 ----
def test_weights_sum_to_one_and_output_is_library_matvec():
    """Sec. 3.4 / Eq. 12-13: sum gamma = 1 and out = G^T gamma."""
    N, d = 11, 70000
    G = _randG(N, d, sigma=2.5)
    st = _state(N)
    for _ in range(3):
        out, info = o.aggregate(G, st)
        assert abs(info["gamma"].sum() - 1.0) <= 1e-12
        assert np.allclose(out, G.astype(np.float64).T @ info["gamma"], rtol=1e-12, atol=1e-14)
        G = _randG(N, d, sigma=2.5)


def test_weighted_sum_row_order_and_bf16():
    """out[k] = sum_i gamma_i G[i,k]: distinct weights on distinct rows (no transposition)."""
    G = np.array([[1, 2, 3], [10, 20, 30]], dtype=np.float32)
    assert np.array_equal(o.weighted_sum(G, [2.0, -1.0]), [-8.0, -16.0, -24.0])
    bits = _to_bf16_bits(_randG(3, 1000))
    gam = np.array([0.5, 0.25, -1.0])
    assert np.allclose(o.weighted_sum(bits, gam), _bf16_bits_to_f64(bits).T @ gam, rtol=1e-14)
    idx = np.array([0, 999, 17, 17])
    assert np.array_equal(o.weighted_sum_at(bits, gam, idx), o.weighted_sum(bits, gam)[idx])


def test_identical_gradients_reduce_to_averaging():
    """Sec. 3.2: equal g_i give the standard average; from zero state gamma = 1/N exactly-ish,
    and with any state the output is still g because the weights sum to one."""
    N, d = 8, 1234
    g = RNG.standard_normal(d).astype(np.float32)
    G = np.tile(g, (N, 1))
    out, info = o.aggregate(G, _state(N))
    assert np.allclose(info["gamma"], 1.0 / N, rtol=1e-13)
    assert np.allclose(out, g.astype(np.float64), rtol=1e-13)
    st = _state(N, beta=0.7)
    for _ in range(4):
        o.aggregate(_randG(N, d, sigma=3.0), st, want_out=False)
    out2, _ = o.aggregate(G, st)
    assert np.allclose(out2, g.astype(np.float64), rtol=1e-12, atol=1e-14)


def test_orthogonal_equal_norm_gradients_get_uniform_weights():
    N = 4
    G = (3.0 * np.eye(N, 16)).astype(np.float32)
    _, info = o.aggregate(G, _state(N), want_out=False)
    assert np.allclose(info["gamma"], 0.25, rtol=1e-14)


@pytest.mark.parametrize("N", [65, 100, 128])
def test_many_workers_keep_the_same_pins(N):
    """The paper's regression runs use up to 128 workers (Appendix A); nothing in the oracle depends on
    N, and the library routines, invariants and special cases pin it there as at small N: K against
    matmul, the output against a matrix-vector product with weights that sum to one, identical
    gradients (Sec. 3.2), orthogonal equal-norm gradients, and worker permutation with a carried state
    (Sec. 3.4)."""
    d = 700
    G = _randG(N, d, sigma=2.0)
    K = o.gram(G)
    assert np.allclose(K, G.astype(np.float64) @ G.astype(np.float64).T, rtol=1e-12, atol=1e-9)
    st_a, st_b = _state(N, beta=0.9), _state(N, beta=0.9)
    for t in range(4):
        G = _randG(N, d, sigma=2.0)
        perm = RNG.permutation(N)
        out_a, info_a = o.aggregate(G, st_a)
        out_b, info_b = o.aggregate(G[perm], st_b)
        assert abs(info_a["gamma"].sum() - 1.0) <= 1e-12
        assert np.allclose(out_a, G.astype(np.float64).T @ info_a["gamma"], rtol=1e-11, atol=1e-12)
        assert np.allclose(info_b["gamma"], info_a["gamma"][perm], rtol=1e-10)
        assert np.allclose(out_b, out_a, rtol=1e-8, atol=1e-11)
    g = RNG.standard_normal(d).astype(np.float32)
    out, info = o.aggregate(np.tile(g, (N, 1)), _state(N))
    assert np.allclose(info["gamma"], 1.0 / N, rtol=1e-12) and np.allclose(out, g.astype(np.float64), rtol=1e-12)
    _, info = o.aggregate((2.0 * np.eye(N, N + 3)).astype(np.float32), _state(N), want_out=False)
    assert np.allclose(info["gamma"], 1.0 / N, rtol=1e-13)


def test_single_worker_and_two_worker_closed_form():
    g = RNG.standard_normal((1, 33)).astype(np.float32)
    out, info = o.aggregate(g, _state(1))
    assert info["gamma"][0] == 1.0 and np.array_equal(out, g[0].astype(np.float64))
    # N = 2: c_1 = (q_1 + p) / (2 q_1), c_2 = (q_2 + p) / (2 q_2), p = <g_1, g_2>
    G = _randG(2, 100, sigma=1.0)
    G[1] *= 3.0
    G64 = G.astype(np.float64)
    q1, q2, p = G64[0] @ G64[0], G64[1] @ G64[1], G64[0] @ G64[1]
    c = np.array([(q1 + p) / (2 * q1), (q2 + p) / (2 * q2)])
    _, info = o.aggregate(G, _state(2), want_out=False)
    assert np.allclose(info["gamma"], c / c.sum(), rtol=1e-12)
    _, info = o.aggregate(G, _state(2, mom=False, norm=False), want_out=False)
    assert np.allclose(info["gamma"], c, rtol=1e-12)


def test_global_rescale_leaves_weights_and_scales_output():
    N, d = 5, 3000
    G = _randG(N, d)
    out1, i1 = o.aggregate(G, _state(N))
    out2, i2 = o.aggregate((G * np.float32(8.0)), _state(N))     # power of two: exact in fp32
    assert np.allclose(i1["gamma"], i2["gamma"], rtol=1e-13)
    assert np.allclose(out2, 8.0 * out1, rtol=1e-13)


def test_larger_gradient_scale_gets_smaller_weight():
    """C2-style heterogeneity: g_i = kappa_i (s + n_i) has c_i ~ (S + kappa_i) / (2 N kappa_i)
    in the large-d limit, S = sum kappa."""
    N, d = 8, 400000
    kappa = 1.0 + 0.1 * np.arange(N)
    G = (_randG(N, d, sigma=1.0) * kappa[:, None]).astype(np.float32)
    _, info = o.aggregate(G, _state(N), want_out=False)
    c = (kappa.sum() + kappa) / (2 * N * kappa)
    assert np.allclose(info["gamma"], c / c.sum(), rtol=2e-2)
    assert (np.diff(info["gamma"]) < 0).all()


def test_adversarial_worker_gets_negative_weight():
    """Consensus behaviour (Sec. 3.2): 15 workers s + n, one -5 s + n.  Large-d limit:
    c = 11/32 for a normal worker, -49/416 for the outlier."""
    N, d = 16, 300000
    s = RNG.standard_normal(d)
    G = s[None, :] + RNG.standard_normal((N, d))
    G[5] = -5.0 * s + RNG.standard_normal(d)
    _, info = o.aggregate(G.astype(np.float32), _state(N), want_out=False)
    c = np.full(N, 11 / 32)
    c[5] = -49 / 416
    assert np.allclose(info["gamma"], c / c.sum(), atol=2e-3)
    assert np.argmin(info["gamma"]) == 5 and info["gamma"][5] < 0
    assert abs(info["gamma"].sum() - 1) < 1e-12


# ------------------------------------------------------------- degenerate ----
def test_zero_gradient_row_is_flagged_and_gets_zero_weight():
    N, d = 4, 64
    G = _randG(N, d)
    G[2] = 0
    out, info = o.aggregate(G, _state(N))
    assert info["numeric_flags"] & o.NUM_ZERO_NORM
    assert info["gamma"][2] == 0.0 and abs(info["gamma"].sum() - 1) < 1e-12
    assert np.isfinite(out).all()


def test_all_zero_and_cancelling_inputs_fall_back_to_uniform():
    st = _state(3)
    out, info = o.aggregate(np.zeros((3, 10), np.float32), st)
    assert info["numeric_flags"] & o.NUM_UNIFORM_FALLBACK
    assert np.allclose(info["gamma"], 1 / 3) and not out.any()
    g = RNG.standard_normal(10).astype(np.float32)
    _, info = o.aggregate(np.stack([g, -g]), _state(2), want_out=False)   # c = 0, 0
    assert info["numeric_flags"] & o.NUM_UNIFORM_FALLBACK
    assert np.allclose(info["gamma"], 0.5)


def test_non_finite_input_falls_back_and_keeps_state():
    N, d = 4, 32
    st = _state(N, beta=0.5)
    o.aggregate(_randG(N, d), st, want_out=False)
    m_before = st.m.copy()
    G = _randG(N, d)
    G[1, 3] = np.inf
    _, info = o.aggregate(G, st, want_out=False)
    assert info["numeric_flags"] & o.NUM_NONFINITE
    assert info["numeric_flags"] & o.NUM_UNIFORM_FALLBACK
    assert np.allclose(info["gamma"], 0.25)
    assert np.array_equal(st.m, m_before) and st.t == 2


def test_threads_do_not_change_the_result(monkeypatch):
    """Chunk-ordered reduction: the result does not depend on the OpenMP thread count."""
    import subprocess, sys, os, json
    code = ("import sys, json, numpy as np; sys.path.insert(0, %r);"
            "from oracle import adacons_oracle as o;"
            "rng = np.random.default_rng(3); G = rng.standard_normal((5, 300001)).astype(np.float32);"
            "print(json.dumps(o.gram(G).ravel().tolist()))") % os.path.dirname(os.path.dirname(__file__))
    outs = []
    for nt in ("1", "5"):
        env = dict(os.environ, OMP_NUM_THREADS=nt)
        outs.append(json.loads(subprocess.check_output([sys.executable, "-c", code], env=env)))
    assert outs[0] == outs[1]


def test_stored_trace_of_the_oracle_itself():
    """Regression guard: the six-step trace written by tests/golden/make_oracle_trace.py (which
    calls only the oracle, on an explicitly specified integer sequence) is reproduced."""
    import importlib.util, os
    here = os.path.dirname(os.path.abspath(__file__))
    spec = importlib.util.spec_from_file_location("make_oracle_trace", os.path.join(here, "golden", "make_oracle_trace.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    stored = np.loadtxt(os.path.join(here, "golden", "oracle_trace_n5_d97.txt"))
    assert stored.shape == (6, 23)
    assert np.allclose(mod.trace(), stored, rtol=1e-13, atol=1e-15)
    assert np.allclose(stored[:, 10:15].sum(axis=1), 1.0, atol=1e-14)
