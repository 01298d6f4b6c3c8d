"""What "the HIP path agrees with the oracle" means, as pure functions of numpy arrays.

The GPU tests hand these functions what the library returned (coefficients, output) together with
what the oracle computed from the same input bits; the CPU tests in test_parity_checks_cpu.py hand
them the oracle's own result with a mistake planted in it and require the check to fail.  Nothing
here touches a GPU.

Tolerances (stated by the benchmark definition): coefficients 1e-6 relative, `out` relative L2
error 1e-5 for fp32 inputs and 2e-3 for bf16 inputs.  On top of the norm, every element of `out`
is held to the rounding bound of the fp32 sum the kernel forms (see assert_out_elementwise).

The sort of Eq. 11 is a discrete decision taken on floating-point values.  Both sides take it in
fp64 on their own first-order coefficients; when the two orders agree (always, unless two
coefficients are closer than the arithmetic error) everything is compared one to one ("strict").
When they differ, the pairs that differ must be ties within 1e-9, and then only what is unique is
compared: the first-order coefficients, the updated state (the EMA acts on the order statistics,
which a tie does not change), that every worker received the state entry of its own rank, that the
weights follow from those entries by the column normalisation and sum to one, and stage A3 against
the oracle's weighted sum of the weights the GPU chose.
"""
import numpy as np

from oracle import adacons_oracle as o

GAMMA_TOL = 1e-6
OUT_TOL = {"f32": 1e-5, "bf16": 2e-3}
U32 = 2.0 ** -24          # unit roundoff of fp32
TIE_TOL = 1e-9


def rel_l2(x, ref):
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.linalg.norm(ref)
    return np.linalg.norm(x - ref) / den if den > 0 else np.linalg.norm(x)


def dtype_name(G) -> str:
    """'f32' or 'bf16' from an oracle input array (float32, or uint16 bit patterns)."""
    return "f32" if np.asarray(G).dtype == np.float32 else "bf16"


def assert_vec_close(got, ref, tol=GAMMA_TOL, what=""):
    """Relative L2 and component-wise (components below 1e-3 of the largest are measured against that floor)."""
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.isfinite(got).all(), (what, got)
    assert rel_l2(got, ref) <= tol, (what, got, ref)
    scale = np.maximum(np.abs(ref), 1e-3 * np.abs(ref).max())
    scale = np.where(scale > 0, scale, 1.0)
    assert (np.abs(got - ref) / scale).max() <= tol, (what, got, ref)


def stable_ranks(a) -> np.ndarray:
    """rank_i = position of worker i in the ascending order of a, ties to the lower index."""
    order = np.argsort(np.asarray(a, dtype=np.float64), kind="stable")
    ranks = np.empty(len(order), dtype=np.int64)
    ranks[order] = np.arange(len(order))
    return ranks


def check_coefficients(info, oinfo, m_after, flags, state_was_zero, ties_possible=False) -> bool:
    """Compare one step's coefficients.  info: what the library returned (gamma, raw, smoothed,
    numeric_flags); oinfo: the oracle's dict for the same input (with "K"); m_after: the oracle's
    state after this step (sorted order); state_was_zero: the state held only zeros before the step.
    Returns True when the comparison was one to one.  With ties_possible False a step whose two
    orders differ is a failure (continuous inputs have no ties)."""
    assert info["numeric_flags"] == oinfo["numeric_flags"], (info["numeric_flags"], oinfo["numeric_flags"])
    fallback = bool(oinfo["numeric_flags"] & (o.NUM_NONFINITE | o.NUM_UNIFORM_FALLBACK))
    sorted_ema = bool(flags & o.FLAG_MOMENTUM) and not (flags & o.FLAG_INDEX_EMA)
    nonfinite = bool(oinfo["numeric_flags"] & o.NUM_NONFINITE)
    if nonfinite:
        # the statistics are poisoned: weights are 1/N, the coefficients carry NaN/Inf on both sides
        N = len(oinfo["gamma"])
        assert np.array_equal(info["gamma"], np.full(N, 1.0 / N)), info["gamma"]
        return True
    assert_vec_close(info["raw"], oinfo["raw"], what="raw")
    rg, rr = stable_ranks(info["raw"]), stable_ranks(oinfo["raw"])
    same_order = np.array_equal(rg, rr)
    # from a zero state every entry receives (1 - beta) a_i whatever its rank: the order cannot matter yet
    strict = (not sorted_ema) or same_order or state_was_zero
    if not strict:
        assert ties_possible, ("the two sides sorted differently on continuous input", info["raw"], oinfo["raw"])
        ref = np.asarray(oinfo["raw"], dtype=np.float64)
        amax = np.abs(ref).max()
        for i in np.nonzero(rg != rr)[0]:
            # worker i sits at another rank: every worker between its two positions must be tied with it
            lo, hi = sorted((rg[i], rr[i]))
            between = np.nonzero((rr >= lo) & (rr <= hi))[0]
            assert np.abs(ref[between] - ref[i]).max() <= TIE_TOL * amax, ("orders differ beyond a tie", i, ref)
    if strict:
        assert_vec_close(info["smoothed"], oinfo["smoothed"], what="smoothed")
        assert_vec_close(info["gamma"], oinfo["gamma"], what="gamma")
        return True
    # a tie broken the other way: compare what is unique, check that the rest is valid
    assert_vec_close(np.sort(info["smoothed"]), np.sort(oinfo["smoothed"]), what="smoothed (as a multiset)")
    assert_vec_close(info["smoothed"], np.asarray(m_after)[rg], what="smoothed against the state entry of its own rank")
    q = np.diag(oinfo["K"]) if "K" in oinfo else np.asarray(oinfo["q"])
    with np.errstate(divide="ignore", invalid="ignore"):
        c = np.where(q > 0, np.asarray(info["smoothed"]) / np.sqrt(q), 0.0)
    if fallback:
        N = len(c)
        assert np.array_equal(info["gamma"], np.full(N, 1.0 / N)), info["gamma"]
    elif flags & o.FLAG_NORMALIZE:
        den = np.asarray(info["smoothed"]).sum() if flags & o.FLAG_LAMBDA_EQ13 else c.sum()
        assert_vec_close(info["gamma"], c / den, what="gamma against its own smoothed coefficients")
        if not flags & o.FLAG_LAMBDA_EQ13:
            assert abs(np.sum(info["gamma"]) - 1.0) <= 1e-9
    else:
        assert_vec_close(info["gamma"], c, what="gamma against its own smoothed coefficients")
    return False


def _abs_input(Gh):
    """|G| in the oracle's input form (fp32: exact; bf16 bit patterns: sign bit cleared)."""
    Gh = np.asarray(Gh)
    if Gh.dtype == np.float32:
        return np.abs(Gh)
    return (Gh.view(np.uint16) & np.uint16(0x7FFF)).astype(np.uint16)


def out_error_bound(Gh, gamma, extra_roundings=0):
    """Element-wise bound on |fp32 weighted sum - exact weighted sum| for out_k = sum_i gamma_i G_ik
    formed as the kernel forms it: gamma rounded to fp32 once, then N fused multiply-adds in worker
    order, fp32 accumulator (bf16 inputs widen exactly).  Standard forward bound of a recursive sum:
    (N + 1) u sum_i |gamma_i| |G_ik| to first order, u = 2^-24; one more u of slack for the second
    order terms, plus the smallest normal fp32 for results that underflow."""
    N = np.asarray(Gh).shape[0]
    mag = o.weighted_sum(_abs_input(Gh), np.abs(np.asarray(gamma, dtype=np.float64)))
    return (N + 2 + extra_roundings) * U32 * mag + 1.2e-38, mag


def assert_out_elementwise(out, Gh, gamma_gpu, base=None, lr=None):
    """Every element of `out` against the oracle's float64 weighted sum of the weights the GPU
    applied (its own fp64 gamma), within the rounding bound above.  With base and lr: out is the
    fused descent step base - lr * sum (one more rounding on the result)."""
    got = np.asarray(out, dtype=np.float64)
    assert np.isfinite(got).all(), "non-finite or unwritten elements in out"
    ref = o.weighted_sum(Gh, gamma_gpu)
    bound, mag = out_error_bound(Gh, gamma_gpu)
    if base is not None:
        base = np.asarray(base, dtype=np.float64)
        ref = base - lr * ref
        bound = abs(lr) * bound + U32 * (np.abs(base) + abs(lr) * mag) + 1.2e-38
    err = np.abs(got - ref)
    bad = np.nonzero(err > bound)[0]
    assert bad.size == 0, ("elements of out beyond the fp32 rounding bound", bad[:8], err[bad[:8]], bound[bad[:8]])
    return ref


def check_out(out, Gh, info, oout, strict):
    """`out` of one aggregation: the element-wise bound against the weighted sum of the GPU's own
    weights, and, when the coefficients were compared one to one, the stated relative L2 tolerance
    against the oracle's output."""
    ref_own = assert_out_elementwise(out, Gh, info["gamma"])
    tol = OUT_TOL[dtype_name(Gh)]
    assert rel_l2(out, ref_own) <= tol
    if strict and oout is not None:
        assert rel_l2(out, oout) <= tol
