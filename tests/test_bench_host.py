"""Host-side logic of bench.py that needs no GPU: the memory-traffic figures of the roofline object
come from the rocprofv3 summaries under profiles/, not from numbers typed into the script."""
import glob
import os
import re
import subprocess
import sys

import bench
import workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_workload_has_a_traffic_summary_and_bench_reads_it():
    for name, w in workloads.CONFIGS.items():
        traffic, src = bench.pmc_traffic(name, {})
        assert traffic is not None, name
        assert os.path.exists(os.path.join(ROOT, "profiles", src))
        a1 = w.N * w.d * w.elem_bytes
        a3 = a1 + 4 * w.d
        # what crossed the fabric is at least the algorithmic bytes (C1 fits the caches: exempt) and within 10 % of them
        for stage, alg in (("gram_kernel (A1)", a1), ("wsum_kernel (A3)", a3)):
            assert stage in traffic, (name, stage)
            if name != "C1":
                assert 0.999 * alg <= traffic[stage] <= 1.10 * alg, (name, stage, traffic[stage], alg)


def test_traffic_table_equals_the_figures_printed_in_the_summaries():
    files = sorted(glob.glob(os.path.join(ROOT, "profiles", "*_hbm_traffic_pmc.txt")))
    assert len(files) >= 5
    for path in files:
        text = open(path).read()
        args = re.search(r"^bench_args: (.*)$", text, re.M).group(1).split()
        wl = args[args.index("--workload") + 1]
        tune = {a.split("=")[0]: int(a.split("=")[1]) for i, a in enumerate(args) if i and args[i - 1] == "--tune"}
        traffic, src = bench.pmc_traffic(wl, tune)
        assert src == os.path.basename(path)
        # recompute from the printed lines: mean reading * 1024 * factor of the section the line is in
        total = {}
        factor = None
        for line in text.splitlines():
            m = re.search(r"scale factor ([\d.]+)", line)
            if m:
                factor = float(m.group(1))
            m = re.search(r"^\s+(adacons::\S.*?)\s+n=\s*\d+ mean reading\s+([\d.]+)\s+->\s+([\d.]+) MB per launch \((\d+) B\)", line)
            if m:
                name, reading, mb, nbytes = m.group(1), float(m.group(2)), float(m.group(3)), int(m.group(4))
                assert abs(nbytes / 1e6 - mb) <= 0.006, line
                assert abs(reading * 1024 * factor - nbytes) <= 6e-5 * nbytes + 6000, line
                for stage, keys in bench.STAGE_KERNELS.items():
                    if any(k in name for k in keys):
                        total[stage] = total.get(stage, 0) + nbytes
        assert total == traffic, path


def test_unprofiled_tuning_reports_no_traffic():
    assert bench.pmc_traffic("C2", {"wsum_park_kb": 64}) == (None, None)


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "single-GPU" in r.stderr
