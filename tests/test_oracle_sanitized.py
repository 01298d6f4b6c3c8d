"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only, CPU only).

Every parity claim rests on oracle/adacons_oracle.c, so its pins are run once more against a build
with -fsanitize=address,undefined: an out-of-bounds index, a use after free or an overflow that
happens to give the right numbers would still end the run.  A second build with a planted
allocation mistake shows that the sanitizer is in fact watching.
"""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "adacons_oracle.c")
PINS = os.path.join(ROOT, "tests", "test_oracle_pins.py")


def _build(src, lib):
    subprocess.run(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off",
                    "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
                    "-o", lib, src, "-lm"], check=True)


def _run_pins(lib, select=None, log=None):
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], check=True, capture_output=True, text=True).stdout.strip()
    preload = ":".join(p for p in (os.environ.get("LD_PRELOAD", ""), asan) if p)
    env = dict(os.environ, ADACONS_ORACLE_LIB_OVERRIDE=lib, OMP_NUM_THREADS="2", LD_PRELOAD=preload,
               ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0:abort_on_error=0:exitcode=99"
                            + (":log_path=" + log if log else ""),
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    cmd = [sys.executable, "-m", "pytest", PINS, "-x", "-q", "-p", "no:cacheprovider"]
    if select:
        cmd += ["-k", select]
    return subprocess.run(cmd, env=env, cwd=ROOT, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)


def test_pins_pass_on_the_sanitized_oracle(tmp_path):
    lib = str(tmp_path / "oracle_asan.so")
    _build(SRC, lib)
    r = _run_pins(lib)
    assert r.returncode == 0, r.stdout[-3000:]
    assert "passed" in r.stdout and "ERROR: AddressSanitizer" not in r.stdout and "runtime error" not in r.stdout


def test_the_sanitizer_is_watching(tmp_path):
    """The three work vectors of the coefficient step allocated as two: the third is written out of bounds."""
    text = open(SRC).read()
    old = "double *a = (double *)malloc(sizeof(double) * (size_t)N * 3);"
    assert text.count(old) == 1
    src = str(tmp_path / "short_alloc.c")
    with open(src, "w") as fh:
        fh.write(text.replace(old, "double *a = (double *)malloc(sizeof(double) * (size_t)N * 2);"))
    lib = str(tmp_path / "short_alloc.so")
    _build(src, lib)
    # the report goes to a file: the child's stderr is captured by its own pytest and lost when the
    # sanitizer ends the process
    log = str(tmp_path / "asan_report")
    r = _run_pins(lib, select="sum_to_one or identical or closed_form", log=log)
    assert r.returncode == 99, (r.returncode, r.stdout[-2000:])
    reports = [open(os.path.join(str(tmp_path), f)).read() for f in os.listdir(str(tmp_path)) if f.startswith("asan_report")]
    assert reports and "heap-buffer-overflow" in reports[0] and "oracle_coefficients_from_stats" in reports[0]
