"""AddressSanitizer + UndefinedBehaviorSanitizer runs of the CPU-side C code: the oracle's
brute-force scan (against the ordinary build's results) and the C program that walks the
library's error paths.  Host code only; nothing here touches a GPU."""
import os
import shutil
import subprocess

import numpy as np
import pytest

from oracle import build as obuild
from paper_2506_19852_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-g", "-O1", "-fno-omit-frame-pointer"]
ENV = dict(os.environ, ASAN_OPTIONS="abort_on_error=0:detect_leaks=1:halt_on_error=1", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
ENV.pop("LD_PRELOAD", None)

pytestmark = pytest.mark.skipif(shutil.which("gcc") is None, reason="no C compiler")

SHAPES = [  # f s block sink num den extra qb_begin qb_end
    (8, 256, 64, 1, 1, 1, 0, 0, 32), (5, 200, 128, 1, 1, 1, 0, 0, 8), (40, 2, 8, 0, 1, 1, 0, 0, 10), (1, 1, 128, 1, 1, 1, 0, 0, 1),
    (7, 33, 64, 2, 13, 20, 0, 1, 3), (9, 50, 64, 1, 3, 1, 77, 0, 9), (12, 7, 4, 0, 1, 7, 5, 3, 23), (3, 333, 128, 5, 1, 1, 1, 7, 8),
]


def test_oracle_scan_under_asan_and_ubsan(tmp_path):
    exe = tmp_path / "scan_san"
    subprocess.check_call(["gcc", "-std=c99", *SAN, "-fopenmp", os.path.join(ROOT, "oracle", "mask_scan.c"),
                           os.path.join(ROOT, "tests", "sanitize", "scan_driver.c"), "-o", str(exe)])
    text = "".join(" ".join(str(t) for t in sh) + "\n" for sh in SHAPES)
    r = subprocess.run([str(exe)], input=text, capture_output=True, text=True, env=dict(ENV, OMP_NUM_THREADS="4"), timeout=300)
    assert r.returncode == 0, r.stderr[-3000:]
    assert "ERROR" not in r.stderr and "runtime error" not in r.stderr, r.stderr[-3000:]
    lines = r.stdout.strip().splitlines()
    assert len(lines) == len(SHAPES)
    for sh, line in zip(SHAPES, lines):
        f, s, block, sink, num, den, extra, qb0, qb1 = sh
        total, _, tsum = (int(t) for t in line.split())
        bitmap, want_total = obuild.mask_scan(f, s, block, sink, qb0, qb1, num, den, extra)   # the ordinary build
        assert total == want_total, sh
        nv = f * s
        rows = min(nv, 40)
        want_tm = obuild.token_mask(f, s, sink, nv - rows, nv, np.arange(nv), num, den)
        assert tsum == int(want_tm.sum()), sh


def test_abi_error_paths_under_asan_and_ubsan(tmp_path):
    exe = tmp_path / "abi_san"
    libdir = os.path.dirname(binding.lib_path())
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", *SAN, "-I", os.path.join(ROOT, "include"),
                           os.path.join(ROOT, "tests", "sanitize", "abi_errors.c"), "-o", str(exe), "-L", libdir, "-lradial",
                           f"-Wl,-rpath,{libdir}"])
    # the HIP runtime that libradial links keeps allocations alive until exit: no leak report for those
    env = dict(ENV, ASAN_OPTIONS="detect_leaks=0:halt_on_error=1")
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0 and r.stdout.strip() == "ok", (r.returncode, r.stdout, r.stderr[-3000:])
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-3000:]
