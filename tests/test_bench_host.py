"""Host-side logic of bench.py that needs no GPU: the flop count of a block list, the lookup of
the counter traffic in a committed rocprofv3 summary, and the refusal of more than one GPU."""
import os
import subprocess
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


def test_effective_flops_counts_real_tokens_only():
    # 3 blocks of 4 tokens over N = 10: the last block holds 2 real tokens
    row_ptr = np.array([0, 2, 3, 6], dtype=np.int32)
    col_idx = np.array([0, 2, 1, 0, 1, 2], dtype=np.int32)
    n, block, d, heads = 10, 4, 8, 3
    pairs = 0
    for qb in range(3):
        for kb in col_idx[row_ptr[qb]:row_ptr[qb + 1]]:
            rows = min(n, (qb + 1) * block) - qb * block
            cols = min(n, (kb + 1) * block) - kb * block
            pairs += rows * cols
    assert bench.effective_flops(row_ptr, col_idx, n, block, d, heads) == 4 * d * pairs * heads


NAMES = ("radial_tile.h", "radial_attn_fwd_kernel.h")  # the files a summary says it depends on

SUMMARY = """{digest_line}# rocprofv3 --kernel-trace --stats -- python3 bench.py
kernel                              calls   avg_ms    min_ms    max_ms
radial_fwd_kernel<128, 128, false, false> radial list              4    {ms}    75.469    77.248

radial_fwd_kernel<128, 128, false, false> radial list            FETCH_SIZE                     avg/launch 2.0e+08
copy probe (torch.neg): FETCH_SIZE 500000 KiB
radial_fwd_kernel<128, 128, false, false> radial list            WRITE_SIZE                     avg/launch 1.0e+06
copy probe: WRITE_SIZE 1000000 KiB
"""


def write_summary(tmp_path, monkeypatch, digest, ms="76.000"):
    line = "" if digest is None else f"# kernel sources at capture (sha256, first 16 hex digits, of {' '.join(NAMES)}): {digest}\n"
    (tmp_path / "fwd_wl.txt").write_text(SUMMARY.format(digest_line=line, ms=ms))
    monkeypatch.setattr(bench, "PROFILES", str(tmp_path))


def test_traffic_scaled_by_the_copy_probe(tmp_path, monkeypatch):
    write_summary(tmp_path, monkeypatch, bench.kernel_source_digest(NAMES))
    copy_bytes = 1000000 * 1024.0  # the copy moved 1e6 KiB each way: fetch counter read half, write counter all
    got, src = bench.traffic_from_profile("wl", 80.0, copy_bytes)  # 5 % slower box: still the same kernel
    assert got == pytest.approx((2.0e8 * 2.0 + 1.0e6 * 1.0) * 1024.0)
    assert src["fetch_scale"] == 2.0 and src["write_scale"] == 1.0 and src["kernel_ms_at_capture"] == 76.0


def test_traffic_is_null_for_other_kernel_sources(tmp_path, monkeypatch):
    write_summary(tmp_path, monkeypatch, "0123456789abcdef")
    got, src = bench.traffic_from_profile("wl", 76.0, 1e9)
    assert got is None and "sources" in src["note"]


def test_traffic_is_null_far_from_the_captured_time(tmp_path, monkeypatch):
    write_summary(tmp_path, monkeypatch, bench.kernel_source_digest(NAMES))
    assert bench.traffic_from_profile("wl", 95.0, 1e9)[0] is None
    write_summary(tmp_path, monkeypatch, None)            # a summary without digest: 3 % rule
    assert bench.traffic_from_profile("wl", 77.0, 1e9)[0] is not None
    assert bench.traffic_from_profile("wl", 80.0, 1e9)[0] is None


def test_traffic_is_null_without_a_summary(tmp_path, monkeypatch):
    monkeypatch.setattr(bench, "PROFILES", str(tmp_path))
    got, src = bench.traffic_from_profile("wl", 76.0, 1e9)
    assert got is None and "no counter summary" in src["note"]


def test_committed_summaries_hold_every_figure_bench_reads():
    for wl in ("cfg3_hunyuan720p", "cfg5_wan480p_4x_bwd"):
        _, src = bench.traffic_from_profile(wl, 1.0, 1e9)   # the time is far off on purpose: only parsing is checked
        assert src["kernel_ms_at_capture"] is not None and src.get("note") != "summary lacks a figure", (wl, src)


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "one GPU" in r.stderr
