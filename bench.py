#!/usr/bin/env python3
"""Benchmark of the AdaCons aggregation hot path on one MI355X.

A step is one whole aggregation (stage A1 Gram, A2 coefficients, A3 weighted sum) through the
C ABI over one N x d gradient matrix already resident in HBM.  The default workload is the
graded one: N = 8 workers, d = 25,557,032 fp32 (ResNet-50-sized), synthetic gradients from the
seeded recipe in workloads/ (two consecutive steps of the stream, used alternately).

Prints ONE JSON line.  `value` is the effective bandwidth: algorithmic bytes of one aggregation
(G read twice + fp32 out written once) divided by the mean time of a step.  Excluded from the
timed region: input generation, host/device copies, coefficient readback.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0   # MI355X published HBM3E peak

PROFILES = os.path.join(ROOT, "profiles")
# kernels of each stage, as rocprofv3 names them
STAGE_KERNELS = {"gram_kernel (A1)": ("gram_", "stats_wave", "stats_edge"), "wsum_kernel (A3)": ("wsum_",)}


def pmc_traffic(workload: str, tuned: dict):
    """Bytes per launch that crossed the L2 <-> memory fabric (fetched + written), per stage, read
    from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summary under profiles/ that was made with this
    workload and tuning (its `bench_args:` line says which).  Returns ({stage: bytes}, file name), or
    (None, None) when no summary covers the configuration: the counters cannot be collected from
    inside a timed run, so a configuration nobody profiled reports null."""
    import glob
    import re
    want = (workload, tuple(sorted((k, int(v)) for k, v in tuned.items() if k != "graph_calls")))
    for path in sorted(glob.glob(os.path.join(PROFILES, "*_hbm_traffic_pmc.txt"))):
        text = open(path).read()
        m = re.search(r"^bench_args: (.*)$", text, re.M)
        if not m:
            continue
        words = m.group(1).split()
        wl = words[words.index("--workload") + 1] if "--workload" in words else "C2"
        tune = tuple(sorted((w.split("=")[0], int(w.split("=")[1]))
                            for i, w in enumerate(words) if i > 0 and words[i - 1] == "--tune"))
        if (wl, tune) != want:
            continue
        per_stage = {}
        for name, nbytes in re.findall(r"^\s+(adacons::\S.*?)\s+n=\s*\d+ mean reading .*\((\d+) B\)\s*$", text, re.M):
            for stage, keys in STAGE_KERNELS.items():
                if any(k in name for k in keys):
                    per_stage[stage] = per_stage.get(stage, 0) + int(nbytes)
        return per_stage, os.path.basename(path)
    return None, None


def cpu_model() -> str:
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="C2", choices=["C1", "C2", "C3", "C4", "C5", "E14"],
                    help="C1..C5: the five configurations (C2 is the one the metric is quoted on); E14: the shape of the\n"
                         "paper's linear-regression example, N = 128, d = 1000 (launch-bound)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--graph", type=int, default=0, metavar="CALLS",
                    help="time the aggregation replayed from a HIP graph that holds CALLS consecutive calls "
                         "(launch-bound small workloads); steps is rounded to a multiple of CALLS")
    ap.add_argument("--no-ceilings", action="store_true",
                    help="skip the read-only and copy rates measured on this box for context")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="REPS",
                    help="after the timed region, run REPS plain device copies of G (known size) so that a "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE run can be scaled to bytes")
    ap.add_argument("--layers", choices=["resnet50"], default=None,
                    help="time the layer-wise entry point instead (C2 or C4): one coefficient set per "
                         "parameter tensor of a ResNet-50; not the headline metric")
    ap.add_argument("--tune", action="append", default=[], metavar="KEY=VALUE",
                    help="gram_blocks_per_cu / wsum_blocks_per_cu / cached_head_mb / gram_products / stats_only / "
                         "wsum_park_kb / short_path")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is a single-GPU hot path; run it with --gpus 1 "
              "(no collectives or sharding are part of it)", file=sys.stderr)
        return 2

    import torch
    import workloads
    import paper_2411_03742_amd as ada

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 3
    dev = "cuda:0"
    torch.cuda.set_device(0)
    w = workloads.CONFIGS.get(args.workload) or workloads.EXTRA[args.workload]

    # two consecutive steps of the seeded stream, kept resident and used alternately
    bufs = []
    for G in workloads.stream(w.scaled(w.d, 2), dev):
        bufs.append(G.clone())
    out = torch.empty(w.d, dtype=torch.float32, device=dev)
    if args.layers:
        return bench_layers(args, w, bufs, out)
    agg = ada.AdaCons(w.N, w.d, beta=0.99)
    keys = {"gram_blocks_per_cu": ada.ADACONS_TUNE_GRAM_BLOCKS_PER_CU,
            "wsum_blocks_per_cu": ada.ADACONS_TUNE_WSUM_BLOCKS_PER_CU,
            "cached_head_mb": ada.ADACONS_TUNE_CACHED_HEAD_MB,
            "gram_products": ada.ADACONS_TUNE_GRAM_PRODUCTS,
            "stats_only": ada.ADACONS_TUNE_STATS_ONLY,
            "wsum_park_kb": ada.ADACONS_TUNE_WSUM_PARK_KB,
            "short_path": ada.ADACONS_TUNE_SHORT_PATH,
            "wsum_row_slices": ada.ADACONS_TUNE_WSUM_ROW_SLICES}
    tuned = {}
    for kv in args.tune:
        k, v = kv.split("=")
        agg.tune(keys[k], int(v))
        tuned[k] = int(v)

    stream = torch.cuda.current_stream()
    # what this machine delivers for a read-only stream and a copy of the same buffers (context for the roofline
    # fraction): measured first, ahead of the warm-up steps
    ceilings = measured_ceilings(w, bufs, out, stream) if not args.no_ceilings else None
    for i in range(args.warmup):
        agg.aggregate(bufs[i % 2], out=out, stream=stream)
    torch.cuda.synchronize()

    # ---- timed region: exactly `steps` aggregations, nothing else on the stream ----------
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    graph = None
    if args.graph > 0:
        # the library enqueues kernels only, so the calls can be captured once and replayed
        args.steps = max(args.graph, args.steps // args.graph * args.graph)
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for i in range(args.graph):
                agg.aggregate(bufs[i % 2], out=out, stream=torch.cuda.current_stream())
        for _ in range(3):
            graph.replay()
        torch.cuda.synchronize()
        tuned["graph_calls"] = args.graph
    t0 = time.perf_counter()
    e0.record(stream)
    if graph is not None:
        for _ in range(args.steps // args.graph):
            graph.replay()
    else:
        for i in range(args.steps):
            agg.aggregate(bufs[i % 2], out=out, stream=stream)
    e1.record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    ms_per_step = max(wall_ms, e0.elapsed_time(e1)) / args.steps
    info = agg.coeffs()
    assert abs(info["gamma"].sum() - 1.0) < 1e-6 and info["numeric_flags"] == 0

    # ---- same loop again with the library's HIP events around each stage (same stream) ----
    nprof = min(args.steps, 1000)
    agg.profile_begin(nprof)
    for i in range(nprof):
        agg.aggregate(bufs[i % 2], out=out, stream=stream)
    prof = agg.profile_end(stream=stream)

    # What an event pair measures with nothing between its two records, on the same stream: the part of
    # every bracketed stage time that is not the kernel (4.4 us on the boxes this ran on; with it taken
    # off, the stage times agree with the kernel durations rocprofv3 reports to about a microsecond).
    pairs0 = [torch.cuda.Event(enable_timing=True) for _ in range(202)]
    for e in pairs0:
        e.record(stream)
    torch.cuda.synchronize()
    gaps = sorted(pairs0[i].elapsed_time(pairs0[i + 1]) for i in range(1, 201))
    bracket_ms = gaps[len(gaps) // 2]

    floor = w.floor_bytes
    gbps = floor / (ms_per_step * 1e-3) / 1e9
    eb = w.elem_bytes
    net = lambda ms: max(ms - bracket_ms, 0.5 * ms)
    stages = {
        "gram_kernel (A1)": (w.N * w.d * eb, net(prof["gram_ms"])),
        "wsum_kernel (A3)": (w.N * w.d * eb + 4 * w.d, net(prof["wsum_ms"])),
    }
    dom = max(stages, key=lambda k: stages[k][1])
    dom_bytes, dom_ms = stages[dom]
    achieved = dom_bytes / (dom_ms * 1e-3) / 1e9
    traffic, traffic_file = pmc_traffic(args.workload, tuned)
    dom_bracketed_ms = prof["gram_ms"] if dom.startswith("gram") else prof["wsum_ms"]
    roofline = {
        "bound": "hbm", "kernel": dom, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBPS, 4),
        "traffic": traffic.get(dom) if traffic else None,
        "traffic_source": ("profiles/" + traffic_file) if traffic else None,
        "algorithmic_bytes_per_launch": dom_bytes, "avg_launch_ms": round(dom_ms, 5),
        # the same fraction from the stage time as bracketed by its two events, empty-bracket time not taken off
        "frac_as_bracketed": round(dom_bytes / (dom_bracketed_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
        "event_bracket_ms": round(bracket_ms, 5),
        "stages_ms": dict({k: round(v[1], 5) for k, v in stages.items()}, **{"finish_kernel (A2)": round(net(prof["coeff_ms"]), 5)}),
        "stages_ms_as_bracketed": {"gram_kernel (A1)": round(prof["gram_ms"], 5), "wsum_kernel (A3)": round(prof["wsum_ms"], 5),
                                   "finish_kernel (A2)": round(prof["coeff_ms"], 5)},
        "stages_GBps": {k: round(v[0] / (v[1] * 1e-3) / 1e9, 1) for k, v in stages.items()},
    }

    # ---- per-call spread: each call bracketed by its own event pair (separate from the timed region:
    # an event record costs a few microseconds on the stream) -------------------------------------
    ncall = min(args.steps, 200)
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(ncall)]
    for i, (a, b) in enumerate(pairs):
        a.record(stream)
        agg.aggregate(bufs[i % 2], out=out, stream=stream)
        b.record(stream)
    torch.cuda.synchronize()
    per_call = sorted(a.elapsed_time(b) for a, b in pairs)
    pct = lambda q: round(per_call[min(ncall - 1, int(q * ncall))], 5)
    per_call_ms = {"p10": pct(0.10), "p50": pct(0.50), "p90": pct(0.90), "calls": ncall}

    if args.copy_calibration > 0:
        scratch = torch.empty_like(bufs[0])
        for _ in range(args.copy_calibration):
            scratch.copy_(bufs[0])          # reads and writes N*d*elem bytes each
        torch.cuda.synchronize()
        del scratch

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(w, bufs[0])

    line = {
        "metric": "aggregation effective HBM bandwidth (N=%d, d=%d, %s): algorithmic bytes per aggregation / time"
                  % (w.N, w.d, w.dtype),
        "value": round(gbps, 1), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": "%s: N=%d workers, d=%d %s gradients, beta=0.99, momentum+normalisation"
                               % (w.name, w.N, w.d, w.dtype), "tuning": tuned},
        "pct_of_hbm_peak": round(100.0 * gbps / HBM_PEAK_GBPS, 2),
        "aggregations_per_s": round(1e3 / ms_per_step, 1),
        "gradients_per_s": round(w.N * 1e3 / ms_per_step, 1),
        "algorithmic_bytes_per_step": floor,
        "per_call_ms": per_call_ms,
        "measured_ceilings": ceilings,
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(line))
    agg.close()
    return 0


def bench_layers(args, w, bufs, out) -> int:
    """Layer-wise aggregation over the 161 parameter tensors of a ResNet-50 (same bytes as C2)."""
    import numpy as np
    import torch
    import workloads
    import paper_2411_03742_amd as ada

    if w.d != sum(workloads.resnet50_layer_sizes()):
        print("bench.py: --layers resnet50 goes with a workload of d = 25,557,032 (C2 or C4)", file=sys.stderr)
        return 2
    off = np.concatenate([[0], np.cumsum(workloads.resnet50_layer_sizes())]).astype(np.int64)
    agg = ada.AdaConsLayers(w.N, off, beta=0.99)
    stream = torch.cuda.current_stream()
    for i in range(args.warmup):
        agg.aggregate(bufs[i % 2], out=out, stream=stream)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record(stream)
    for i in range(args.steps):
        agg.aggregate(bufs[i % 2], out=out, stream=stream)
    e1.record(stream)
    torch.cuda.synchronize()
    ms = max((time.perf_counter() - t0) * 1e3, e0.elapsed_time(e1)) / args.steps
    gam = agg.coeffs()["gamma"]
    assert np.abs(gam.sum(axis=1) - 1.0).max() < 1e-6
    gbps = w.floor_bytes / (ms * 1e-3) / 1e9
    print(json.dumps({
        "metric": "layer-wise aggregation effective HBM bandwidth (N=%d, d=%d, %s, %d layers)" % (w.N, w.d, w.dtype, len(off) - 1),
        "value": round(gbps, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": "%s cut into the 161 parameter tensors of a ResNet-50, layer-wise coefficients" % w.name},
        "pct_of_hbm_peak": round(100.0 * gbps / HBM_PEAK_GBPS, 2), "roofline": None, "cpu_baseline": None}))
    agg.close()
    return 0


def measured_ceilings(w, bufs, out, stream) -> dict:
    """Context for the roofline fraction: what this machine delivers for a read-only stream and for a
    plain copy of the same buffers.  Read-only: the library's two-vector statistics kernel
    (adacons_worker_stats: reads two vectors once, writes three doubles) over the two halves of G;
    copy: a device-to-device copy of G (reads and writes N*d elements)."""
    import torch
    import paper_2411_03742_amd as ada

    G = bufs[0]
    half = (w.N // 2) * w.d
    if half < 1:
        return None
    flat = G.reshape(-1)
    x, y = flat[:half], flat[half:2 * half]
    probe = ada.AdaCons(2, half)
    reps = 20
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(3):
        probe.worker_stats(x, y, stream=stream)
    e0.record(stream)
    for _ in range(reps):
        probe.worker_stats(x, y, stream=stream)
    e1.record(stream)
    torch.cuda.synchronize()
    read_gbps = 2 * half * G.element_size() / (e0.elapsed_time(e1) / reps * 1e-3) / 1e9
    probe.close()
    dst = bufs[1]
    for _ in range(3):
        dst.copy_(G)
    e0.record(stream)
    for _ in range(reps):
        dst.copy_(G)
    e1.record(stream)
    torch.cuda.synchronize()
    copy_gbps = 2 * G.numel() * G.element_size() / (e0.elapsed_time(e1) / reps * 1e-3) / 1e9
    return {"read_only_GBps": round(read_gbps, 1), "copy_GBps": round(copy_gbps, 1), "unit": "GB/s",
            "note": "read-only: two-vector statistics kernel over G's halves; copy: device-to-device copy of G "
                    "(bytes read + written)"}


def cpu_baseline(w, G) -> dict:
    """The float64 oracle, as it stands, on this machine's host cores: whole aggregations of the same
    workload (Gram, coefficients, weighted sum), repeated for a bounded time."""
    import numpy as np
    import workloads
    from oracle import adacons_oracle as o

    Gh = workloads.to_oracle_input(G)
    times = []
    budget_s, t_start = 15.0, time.perf_counter()
    st = o.OracleState(w.N, beta=0.99)
    cores = o.num_threads()
    while len(times) < 3 or time.perf_counter() - t_start < budget_s:
        t0 = time.perf_counter()
        o.aggregate(Gh, st, want_out=True)
        times.append(time.perf_counter() - t0)
    med = float(np.median(times))
    # the same oracle on one thread: a single aggregation, or a column prefix of it when the whole
    # input would take more than about ten seconds
    frac = min(1.0, 10.0 / (med * cores))
    d1 = max(1, int(w.d * frac))
    G1 = np.ascontiguousarray(Gh[:, :d1])
    o.set_num_threads(1)
    t0 = time.perf_counter()
    o.aggregate(G1, o.OracleState(w.N, beta=0.99), want_out=True)
    t1 = time.perf_counter() - t0
    o.set_num_threads(cores)
    floor1 = 2 * w.N * d1 * w.elem_bytes + 4 * d1
    return {"value": round(w.floor_bytes / med / 1e9, 3), "unit": "GB/s", "cores": cores,
            "kind": "oracle", "cpu_model": cpu_model(), "host_logical_cpus": os.cpu_count(), "seconds_per_aggregation": round(med, 4),
            "aggregations_per_s": round(1.0 / med, 4),
            "sample": "%d whole aggregations of the full %s input (one step of the stream) in %.0f s, median time"
                      % (len(times), w.name, sum(times)),
            "single_thread": {"value": round(floor1 / t1 / 1e9, 3), "unit": "GB/s", "cores": 1,
                              "sample": "one aggregation of the first %d columns (%.0f %% of the input) in %.1f s"
                                        % (d1, 100.0 * d1 / w.d, t1)}}


if __name__ == "__main__":
    sys.exit(main())
