"""The library called from plain C (tests/c_abi_check.c, built with gcc against include/moe.h):
the program checks fused == staged, permutation and weight invariants, zero in -> zero out and an
error path, and exits non-zero on any failure."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_c_program_runs_the_whole_path():
    exe = os.path.join(ROOT, "paper_2503_09716_amd", "c_abi_check")
    assert os.path.exists(exe), "build first: python paper_2503_09716_amd/build.py"
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    print(r.stdout, r.stderr, flush=True)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "C ABI check passed" in r.stdout
