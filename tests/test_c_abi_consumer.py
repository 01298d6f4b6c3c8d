"""The library driven from a plain-C program (tests/c_abi/roundtrip.c, compiled by build()): no
Python, no torch in the call path.  The program checks closed-form cases itself and reports by exit code."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
EXE = os.path.join(ROOT, "tests", "c_abi", "roundtrip")


@pytest.mark.gpu
def test_plain_c_program_gets_the_closed_form_results():
    if not os.path.exists(EXE):      # normally compiled by __graft_entry__.build(); a one-second hipcc link otherwise
        import __graft_entry__ as entry
        import paper_2411_03742_amd as pkg
        entry.build_c_consumer(pkg.library_path())
    r = subprocess.run([EXE], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
    assert r.returncode == 0, r.stdout
    assert r.stdout.count(": ok") == 4, r.stdout


def test_c_program_source_uses_only_the_public_header():
    text = open(os.path.join(ROOT, "tests", "c_abi", "roundtrip.c")).read()
    assert '#include "adacons.h"' in text and "adacons_internal" not in text and "torch" not in text
