"""adacons_aggregate_noalloc(): the aggregation for callers that cannot allocate device memory.
Same kernels and launch shapes as adacons_aggregate(), its workspace in the library's file-scope
device array, the carried state in the caller's hands.  Checked through the C ABI against
adacons_aggregate() -- bit for bit, both take the same kernels -- on calls in a row that share the
array: the second with a shorter input, then other worker counts, dtypes and the statistics-only
first pass of N > 64, and against the oracle with the shared parity checks."""
import numpy as np
import pytest
import torch

import workloads
from oracle import adacons_oracle as o
from parity_checks import check_coefficients, check_out

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def pkg():
    if not torch.cuda.is_available():
        pytest.fail("these tests need the GPU")
    import paper_2411_03742_amd as p
    return p


def randG(N, d, dtype=torch.float32, sigma=2.0, seed=0):
    g = torch.Generator(device=DEV).manual_seed(seed)
    s = torch.randn(d, generator=g, device=DEV)
    G = s[None, :] + sigma * torch.randn(N, d, generator=g, device=DEV)
    return G.to(dtype).contiguous()


def run_pair(pkg, N, sizes, dtype=torch.float32, beta=0.9, flags=3):
    """The same stream of inputs through adacons_aggregate (own state) and adacons_aggregate_noalloc
    (state in the caller's m); the lengths in `sizes` follow each other on the shared array."""
    ref = pkg.AdaCons(N, max(sizes), beta=beta, flags=flags)
    ost = o.OracleState(N, beta=beta, flags=flags)
    m = torch.zeros(N, dtype=torch.float64, device=DEV)
    coeffs = torch.full((3 * N,), float("nan"), dtype=torch.float64, device=DEV)
    nflags = torch.full((1,), -1, dtype=torch.int32, device=DEV)
    for t, d in enumerate(sizes):
        G = randG(N, d, dtype, seed=1000 * N + t)
        want = ref.aggregate(G).clone()
        winfo = ref.coeffs()
        out = torch.full((d,), float("nan"), dtype=torch.float32, device=DEV)
        pkg.adacons_aggregate_noalloc(G, m, out, beta=beta, flags=flags, coeffs=coeffs, numeric_flags=nflags)
        torch.cuda.synchronize()
        assert torch.equal(out, want), (N, d, t)
        c = coeffs.cpu().numpy().reshape(3, N)
        assert np.array_equal(c[0], winfo["gamma"]) and np.array_equal(c[1], winfo["raw"]) and np.array_equal(c[2], winfo["smoothed"])
        assert int(nflags.item()) == winfo["numeric_flags"]
        m_ref, _ = ref.export_state()
        assert np.array_equal(m.cpu().numpy(), m_ref)
        # and against the oracle, to the same bar as every other entry point
        Gh = workloads.to_oracle_input(G)
        was_zero = not ost.m.any()
        oout, oinfo = o.aggregate(Gh, ost)
        info = {"gamma": c[0], "raw": c[1], "smoothed": c[2], "numeric_flags": int(nflags.item())}
        strict = check_coefficients(info, oinfo, ost.m, ost.flags, was_zero)
        check_out(out.cpu().numpy(), Gh, info, oout, strict)
    ref.close()


def test_two_calls_in_a_row_the_second_smaller(pkg):
    run_pair(pkg, 8, [1_000_004, 300_000, 1_000_004])


@pytest.mark.parametrize("N,sizes,dtype", [(4, [200_003, 4099], torch.float32), (16, [400_000, 65_540], torch.float32),
                                           (64, [150_000, 40_004], torch.float32), (8, [800_008, 100_000], torch.bfloat16),
                                           (100, [60_000, 9_999], torch.float32), (1, [5000, 7], torch.float32)])
def test_other_worker_counts_share_the_array(pkg, N, sizes, dtype):
    run_pair(pkg, N, sizes, dtype)


def test_ablation_flags_and_no_optional_outputs(pkg):
    run_pair(pkg, 8, [100_000, 50_000], flags=0)
    run_pair(pkg, 8, [100_000, 50_000], flags=7)
    N, d = 8, 70_000
    G = randG(N, d, seed=5)
    m = torch.zeros(N, dtype=torch.float64, device=DEV)
    out = torch.empty(d, device=DEV)
    pkg.adacons_aggregate_noalloc(G, m, out)            # coeffs_dev and numeric_flags_dev NULL
    ref = pkg.AdaCons(N, d)
    assert torch.equal(out, ref.aggregate(G))
    ref.close()


def test_sizes_beyond_the_maximum_are_rejected_with_a_message(pkg):
    N, d = 129, 100
    G = torch.zeros(N, d, device=DEV)
    m = torch.zeros(N, dtype=torch.float64, device=DEV)
    with pytest.raises(pkg.AdaConsError) as e:
        pkg.adacons_aggregate_noalloc(G, m, torch.empty(d, device=DEV))
    assert e.value.status == 2 and "maximum" in str(e.value)
    with pytest.raises(pkg.AdaConsError) as e:       # out overlaps G
        G4 = torch.zeros(4, d, device=DEV)
        pkg.adacons_aggregate_noalloc(G4, torch.zeros(4, dtype=torch.float64, device=DEV), G4[3])
    assert e.value.status == 1


def test_it_allocates_nothing_and_can_be_captured(pkg):
    """After a first call (which resolves the array's address), device memory in use does not move
    across further calls, and the call can sit in a HIP graph: replays advance the caller's state."""
    N, d = 8, 500_000
    G = randG(N, d, seed=9)
    m = torch.zeros(N, dtype=torch.float64, device=DEV)
    out = torch.empty(d, device=DEV)
    pkg.adacons_aggregate_noalloc(G, m, out)
    torch.cuda.synchronize()
    free0, _ = torch.cuda.mem_get_info()
    for _ in range(5):
        pkg.adacons_aggregate_noalloc(G, m, out)
    torch.cuda.synchronize()
    free1, _ = torch.cuda.mem_get_info()
    assert free0 == free1
    # graph: three replays against three eager calls on a stateful reference
    m.zero_()
    ref = pkg.AdaCons(N, d)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    m_cap = torch.zeros(N, dtype=torch.float64, device=DEV)
    with torch.cuda.graph(graph, stream=side):
        pkg.adacons_aggregate_noalloc(G, m_cap, out, stream=torch.cuda.current_stream())
    m_cap.zero_()
    for rep in range(3):
        G.copy_(randG(N, d, seed=20 + rep))
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, ref.aggregate(G))
    ref.close()
