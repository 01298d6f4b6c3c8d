"""The pins must notice a plausible mistake anywhere in the oracle.

Each case plants one mistake in a copy of the oracle's C source (a dropped term, a
wrong sign or index, a transposed operand, a wrong exponent), builds it, and runs the
pin tests against that build in a child process: they have to fail.  Everything here
happens on the CPU.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "adacons_oracle.c")

MUTATIONS = [
    ("dot_same_operand", "acc += (double)x[k] * (double)y[k];", "acc += (double)x[k] * (double)x[k];"),
    ("dropped_chunk_offset", "g + (size_t)j * d + k0, len);\n                } else {",
     "g + (size_t)j * d, len);\n                } else {"),
    ("dropped_tail_chunk", "(d + ORACLE_CHUNK - 1) / ORACLE_CHUNK;", "(d < ORACLE_CHUNK) ? 1 : d / ORACLE_CHUNK;"),
    ("bf16_shift", "(uint32_t)h << 16", "(uint32_t)h << 15"),
    ("row_sum_upper_triangle_only", "for (int j = 0; j < N; ++j)\n            acc += K[", "for (int j = i; j < N; ++j)\n            acc += K["),
    ("coefficient_divides_by_squared_norm", "a[i] = r[i] / ((double)N * sqrt(q[i]));", "a[i] = r[i] / ((double)N * q[i]);"),
    ("coefficient_misses_mean", "a[i] = r[i] / ((double)N * sqrt(q[i]));", "a[i] = r[i] / sqrt(q[i]);"),
    ("coefficient_sign", "a[i] = r[i] / ((double)N * sqrt(q[i]));", "a[i] = -r[i] / ((double)N * sqrt(q[i]));"),
    ("sort_descending", "if (a[j] < a[i] || (a[j] == a[i] && j < i))", "if (a[j] > a[i] || (a[j] == a[i] && j < i))"),
    ("ties_to_higher_index", "(a[j] == a[i] && j < i)", "(a[j] == a[i] && j > i)"),
    ("ema_weights_swapped", "m[rank] = beta * m[rank] + (1.0 - beta) * a[i];", "m[rank] = (1.0 - beta) * m[rank] + beta * a[i];"),
    ("ema_not_redistributed_by_rank", "as[i] = m[rank];", "as[i] = m[i];"),
    ("index_coupled_ema", "m[rank] = beta * m[rank] + (1.0 - beta) * a[i];\n            as[i] = m[rank];",
     "m[i] = beta * m[i] + (1.0 - beta) * a[i];\n            as[i] = m[i];"),
    ("second_norm_division_dropped", "c[i] = (q[i] > 0.0) ? as[i] / sqrt(q[i]) : 0.0;", "c[i] = as[i];"),
    ("second_norm_division_squared", "c[i] = (q[i] > 0.0) ? as[i] / sqrt(q[i]) : 0.0;", "c[i] = (q[i] > 0.0) ? as[i] / q[i] : 0.0;"),
    ("normalised_by_abs_sum", "gamma[i] = c[i] / s;", "gamma[i] = c[i] / sabs;"),
    ("weighted_sum_transposed", "acc += gamma[i] * elem(G, dtype, (size_t)i * d + k);\n        out[k] = acc;",
     "acc += gamma[i] * elem(G, dtype, (size_t)k * N + i);\n        out[k] = acc;"),
    ("weighted_sum_drops_first_worker", "for (int i = 0; i < N; ++i)\n            acc += gamma[i] * elem(G, dtype, (size_t)i * d + k);\n        out[k] = acc;",
     "for (int i = 1; i < N; ++i)\n            acc += gamma[i] * elem(G, dtype, (size_t)i * d + k);\n        out[k] = acc;"),
    ("index_ema_weights_swapped", "m[i] = beta * m[i] + (1.0 - beta) * a[i];", "m[i] = (1.0 - beta) * m[i] + beta * a[i];"),
    ("index_ema_still_sorted", "if ((flags & ORACLE_FLAG_MOMENTUM) && (flags & ORACLE_FLAG_INDEX_EMA)) {",
     "if (0) {"),
    ("lambda_eq13_switch_ignored", "(flags & ORACLE_FLAG_LAMBDA_EQ13) ? as : c;", "(flags & ORACLE_FLAG_LAMBDA_EQ13) ? c : c;"),
    ("lambda_eq13_always_on", "(flags & ORACLE_FLAG_LAMBDA_EQ13) ? as : c;", "(flags & ORACLE_FLAG_LAMBDA_EQ13) ? as : as;"),
    ("state_updated_on_non_finite", "nf |= ORACLE_NUM_NONFINITE | ORACLE_NUM_UNIFORM_FALLBACK;",
     "nf |= ORACLE_NUM_NONFINITE | ORACLE_NUM_UNIFORM_FALLBACK; m[0] += 1.0;"),
]


def _run_case(case, tmpdir):
    name, old, new = case
    text = open(SRC).read()
    assert text.count(old) == 1, f"{name}: fragment must occur exactly once (found {text.count(old)})"
    csrc = os.path.join(tmpdir, name + ".c")
    lib = os.path.join(tmpdir, name + ".so")
    with open(csrc, "w") as fh:
        fh.write(text.replace(old, new))
    subprocess.run(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off",
                    "-o", lib, csrc, "-lm"], check=True)
    env = dict(os.environ, ADACONS_ORACLE_LIB_OVERRIDE=lib, OMP_NUM_THREADS="2")
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"),
                        "-x", "-q", "-p", "no:cacheprovider"], env=env, cwd=ROOT,
                       stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    return name, r.returncode, r.stdout[-400:]


def test_every_planted_mistake_fails_a_pin(tmp_path):
    with ThreadPoolExecutor(max_workers=4) as ex:
        results = list(ex.map(lambda c: _run_case(c, str(tmp_path)), MUTATIONS))
    survived = [(n, tail) for n, rc, tail in results if rc == 0]
    assert not survived, f"mutations the pins did not notice: {survived}"
    broken = [(n, rc) for n, rc, _ in results if rc not in (0, 1)]
    assert not broken, f"pin run did not end in an ordinary test failure: {broken}"
