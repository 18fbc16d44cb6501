"""A plain C program drives the library on the GPU through the C ABI (no torch, no ctypes) and
checks the lists and sampled output rows against the oracle's fixture (run with -m gpu)."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_c_program_forward_matches_the_oracle_fixture():
    exe = os.path.join(ROOT, "tests", "abi_gpu", "abi_forward")
    if not os.path.exists(exe):                       # normally built beforehand by __graft_entry__.build()
        import sys
        sys.path.insert(0, os.path.join(ROOT, "tests", "abi_gpu"))
        import build as abi_build
        abi_build.build()
    fixture = os.path.join(ROOT, "tests", "golden", "abi_forward_fixture.txt")
    print("running", exe, flush=True)
    r = subprocess.run([exe, fixture], capture_output=True, text=True, timeout=100)
    print(r.stdout, r.stderr, flush=True)
    assert r.returncode == 0, (r.returncode, r.stdout[-2000:], r.stderr[-2000:])
    assert "16 rows checked" in r.stdout and "lists bit-exact" in r.stdout
