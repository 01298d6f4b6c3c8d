"""Register and scratch budgets of the hot kernels, read from the compiler's own output for this
library's sources (gfx950 cross-compile, no GPU needed).

The launch shapes in the host code assume an occupancy: eight workgroups per CU for the fp32 second pass
of N = 4 and 8 (at most 64 vector registers), two wavefronts per SIMD for the split-bf16 Gram kernel (at
most 256), no spills anywhere on the hot path.  A source change that looks harmless can cost a
register granule and with it a resident wavefront (it did once: 7 % of the second pass); this test
notices at build time."""
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2411_03742_amd", "csrc")
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _kernels(src, tmp_path):
    obj = str(tmp_path / (src + ".o"))
    subprocess.run(["/opt/rocm/bin/hipcc", *FLAGS, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-c",
                    os.path.join(CSRC, src + ".hip"), "-o", obj, "-save-temps=obj"],
                   check=True, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
    text = open(str(tmp_path / (src + "-hip-amdgcn-amd-amdhsa-gfx950.s"))).read()
    out = {}
    for m in re.finditer(r"\.amdhsa_kernel (\S+)(.*?)\.end_amdhsa_kernel", text, re.S):
        body = m.group(2)
        get = lambda k: int(re.search(r"\.amdhsa_" + k + r" (\d+)", body).group(1))
        demangled = subprocess.run(["c++filt", m.group(1)], capture_output=True, text=True).stdout.strip()
        out[demangled.split("(")[0].replace("void ", "")] = {
            "vgpr": get("next_free_vgpr"), "scratch": get("private_segment_fixed_size"), "lds": get("group_segment_fixed_size")}
    return out


def _find(kernels, prefix):
    hits = {k: v for k, v in kernels.items() if k.startswith(prefix)}
    assert hits, (prefix, sorted(kernels)[:5])
    return hits


def test_second_pass_kernels_keep_their_occupancy(tmp_path):
    k = _kernels("wsum", tmp_path)
    for name in ("adacons::wsum_kernel<4, float, 4, 2, false>", "adacons::wsum_kernel<8, float, 4, 2, false>"):
        (res,) = _find(k, name).values()
        assert res["vgpr"] <= 64 and res["scratch"] == 0, (name, res)          # eight wavefronts per SIMD
    for name, res in k.items():
        assert res["scratch"] == 0, (name, res)
    (res,) = _find(k, "adacons::wsum_parked_kernel<16, float, 4, 1, false, 256>").values()
    assert res["vgpr"] <= 128, res                                                 # one workgroup per CU, latency hidden by the tile depth
    for name, res in _find(k, "adacons::wsum_short_kernel<").items():
        assert res["vgpr"] <= 256 and res["lds"] < 16384, (name, res)


def test_first_pass_kernels_keep_their_occupancy(tmp_path):
    k = _kernels("gram", tmp_path)
    for name, res in k.items():
        assert res["scratch"] == 0, (name, res)
    for n in range(1, 9):
        (res,) = _find(k, "adacons::gram_vec_kernel<%d, float, 4, 1>" % n).values()
        assert res["vgpr"] <= 256, (n, res)                                        # two wavefronts per SIMD (launch bound)
    # split-bf16 Gram, two wavefronts per chunk: two wavefronts per SIMD and four workgroups' planes in LDS
    (res,) = _find(k, "adacons::gram_mfma_split_coop_kernel<4, 2>").values()
    assert res["vgpr"] <= 256 and 4 * res["lds"] <= 160 * 1024, res
    (res,) = _find(k, "adacons::gram_mfma_split_coop_kernel<3, 2>").values()
    assert res["vgpr"] <= 168, res


@pytest.mark.parametrize("src", ["stats", "layers", "worker"])
def test_no_kernel_spills(tmp_path, src):
    for name, res in _kernels(src, tmp_path).items():
        assert res["scratch"] == 0, (name, res)
