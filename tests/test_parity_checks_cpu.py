"""The parity checks themselves, tested on the CPU: the oracle's own result stands in for what the
library returned, a mistake is planted in it, and the check has to fail.  Covers the cases the GPU
suite relies on: one-column inputs (every |a_i| tied), a tie broken the other way with a carried
state, a wrong weight, an unwritten tail too short for a norm to see, a single wrong element."""
import numpy as np
import pytest

import parity_checks as pc
from oracle import adacons_oracle as o


def _fp32_out(Gh, gamma):
    """A stand-in for the kernel: gamma rounded to fp32, fp32 fused multiply-adds in worker order
    (emulated in float64: a product of two fp32 values is exact there, one rounding per step)."""
    G = Gh.astype(np.float64) if Gh.dtype == np.float32 else (Gh.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    g32 = np.asarray(gamma, dtype=np.float32).astype(np.float64)
    acc = np.zeros(G.shape[1], dtype=np.float32)
    for i in range(G.shape[0]):
        acc = (acc.astype(np.float64) + g32[i] * G[i]).astype(np.float32)
    return acc


def _step(G, ost):
    was_zero = not ost.m.any()
    oout, oinfo = o.aggregate(G, ost)
    info = {k: np.array(oinfo[k]) for k in ("gamma", "raw", "smoothed")}
    info["numeric_flags"] = oinfo["numeric_flags"]
    return info, oinfo, oout, was_zero


def _rand(N, d, seed, sigma=2.0):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal(d)[None, :] + sigma * rng.standard_normal((N, d))).astype(np.float32)


def test_agreeing_result_passes_and_is_strict():
    ost = o.OracleState(6, beta=0.9)
    for t in range(3):
        G = _rand(6, 5000, t)
        info, oinfo, oout, z = _step(G, ost)
        assert pc.check_coefficients(info, oinfo, ost.m, ost.flags, z)
        pc.check_out(_fp32_out(G, info["gamma"]), G, info, oout, True)


@pytest.mark.parametrize("N", [2, 16, 128])
def test_wrong_weight_on_a_one_column_input_fails(N):
    """d = 1: a_i = sign(x_i) sum(x) / N, all |a_i| tied.  A wrong gamma has to be caught both on the
    first step (zero state: compared one to one) and on a later one (compared through its own
    smoothed coefficients)."""
    rng = np.random.default_rng(N)
    ost = o.OracleState(N, beta=0.8)
    for t in range(3):
        G = rng.standard_normal((N, 1)).astype(np.float32)
        info, oinfo, oout, z = _step(G, ost)
        pc.check_coefficients(info, oinfo, ost.m, ost.flags, z, ties_possible=True)
        pc.check_out(_fp32_out(G, info["gamma"]), G, info, oout, True)
        bad = dict(info, gamma=info["gamma"].copy())
        bad["gamma"][N // 2] *= 1.0 + 5e-6
        with pytest.raises(AssertionError):
            pc.check_coefficients(bad, oinfo, ost.m, ost.flags, z, ties_possible=True)
        # a right gamma applied wrongly in stage A3 is caught by the element-wise bound
        with pytest.raises(AssertionError):
            pc.check_out(_fp32_out(G, bad["gamma"]) * np.float32(1.001), G, info, oout, True)


def test_tie_broken_the_other_way_is_accepted_only_when_it_is_a_tie():
    """Two workers with identical gradients tie exactly.  Handing their two state entries to them in
    the other order is a valid result (the output does not change); the same swap between workers
    that are not tied is not."""
    N, d = 5, 3000
    ost = o.OracleState(N, beta=0.5)
    G = _rand(N, d, 1)
    _step(G, ost)                                   # state now non-zero and not uniform
    G = _rand(N, d, 2)
    G[3] = G[1]
    m_before = ost.m.copy()
    info, oinfo, oout, z = _step(G, ost)
    r = pc.stable_ranks(oinfo["raw"])
    assert abs(r[1] - r[3]) == 1 and oinfo["raw"][1] == oinfo["raw"][3]
    # what a library that broke the tie the other way would return: raw differs in the last bit
    swapped = {k: info[k].copy() for k in ("gamma", "raw", "smoothed")}
    swapped["numeric_flags"] = info["numeric_flags"]
    swapped["raw"][3] = np.nextafter(swapped["raw"][3], -np.inf)       # worker 3 now sorts before worker 1
    swapped["smoothed"][[1, 3]] = info["smoothed"][[3, 1]]
    q = np.diag(oinfo["K"])
    c = swapped["smoothed"] / np.sqrt(q)
    swapped["gamma"] = c / c.sum()
    with pytest.raises(AssertionError):             # continuous inputs: a different order is a failure
        pc.check_coefficients(swapped, oinfo, ost.m, ost.flags, z, ties_possible=False)
    assert pc.check_coefficients(swapped, oinfo, ost.m, ost.flags, z, ties_possible=True) is False
    out = _fp32_out(G, swapped["gamma"])
    pc.check_out(out, G, swapped, oout, False)
    assert pc.rel_l2(out, oout) <= 1e-5             # tied workers hold equal gradients: same output
    # the same exchange between two workers that are NOT tied
    i, j = np.argsort(oinfo["raw"])[[0, N - 1]]
    wrong = {k: info[k].copy() for k in ("gamma", "raw", "smoothed")}
    wrong["numeric_flags"] = info["numeric_flags"]
    wrong["smoothed"][[i, j]] = info["smoothed"][[j, i]]
    with pytest.raises(AssertionError):
        pc.check_coefficients(wrong, oinfo, ost.m, ost.flags, z, ties_possible=True)
    assert m_before.any()


def test_unwritten_tail_and_single_wrong_element_fail_where_a_norm_would_not():
    """bf16 tolerance 2e-3 on the norm: eight unwritten columns out of 8,000,000 are a relative L2 error
    of sqrt(8 / 8e6) = 1e-3 -- invisible to it; the element-wise bound sees them."""
    N, d = 4, 8_000_000
    G = _rand(N, d, 7)
    Gb = (G.view(np.uint32) >> 16).astype(np.uint16)      # truncated to bf16 bit patterns
    ost = o.OracleState(N)
    info, oinfo, oout, z = _step(Gb, ost)
    out = _fp32_out(Gb, info["gamma"])
    pc.check_out(out, Gb, info, oout, True)
    tail = out.copy()
    tail[-8:] = 0.0
    assert pc.rel_l2(tail, oout) <= pc.OUT_TOL["bf16"]    # the norm alone would pass
    with pytest.raises(AssertionError):
        pc.check_out(tail, Gb, info, oout, True)
    one = out.copy()
    one[123_456] *= np.float32(1.0 + 1e-4)
    assert one[123_456] != out[123_456]
    assert pc.rel_l2(one, oout) <= pc.OUT_TOL["bf16"]
    with pytest.raises(AssertionError):
        pc.check_out(one, Gb, info, oout, True)
    nan = out.copy()
    nan[5] = np.nan
    with pytest.raises(AssertionError):
        pc.check_out(nan, Gb, info, oout, True)


def test_fused_descent_step_bound():
    N, d = 4, 10_000
    G = _rand(N, d, 3)
    ost = o.OracleState(N)
    info, oinfo, oout, z = _step(G, ost)
    w0 = np.random.default_rng(0).standard_normal(d).astype(np.float32)
    acc = _fp32_out(G, info["gamma"])
    w1 = (w0.astype(np.float64) - np.float64(np.float32(0.25)) * acc.astype(np.float64)).astype(np.float32)
    pc.assert_out_elementwise(w1, G, info["gamma"], base=w0, lr=0.25)
    with pytest.raises(AssertionError):
        pc.assert_out_elementwise(w0, G, info["gamma"], base=w0, lr=0.25)      # step not applied


def test_flags_mismatch_and_wrong_raw_fail():
    ost = o.OracleState(4)
    G = _rand(4, 100, 5)
    info, oinfo, oout, z = _step(G, ost)
    with pytest.raises(AssertionError):
        pc.check_coefficients(dict(info, numeric_flags=1), oinfo, ost.m, ost.flags, z)
    bad = dict(info, raw=info["raw"] * (1 + 3e-6))
    with pytest.raises(AssertionError):
        pc.check_coefficients(bad, oinfo, ost.m, ost.flags, z)
