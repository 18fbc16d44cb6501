"""Writes tests/golden/block_counts.txt from the oracle's full brute-force scan (calls only oracle/).

Per workload and sink setting: listed block pairs, shortest / longest list, an order-sensitive
checksum of the compressed list, and the visible-token-pair count.  Run from the repo root:
    python tests/golden/make_block_counts.py
(the 464 400-token workload scans 2.2e11 token pairs: minutes)."""
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import build as obuild  # noqa: E402
from oracle import mask as om  # noqa: E402

# name, frames, tokens per frame, block (the five workload shapes)
SHAPES = [("cfg1_tiny", 8, 256, 64), ("cfg2_wan480p", 21, 1560, 128), ("cfg3_hunyuan720p", 33, 3600, 128),
          ("cfg4_hunyuan720p_4x", 129, 3600, 128), ("cfg5_wan480p_4x_bwd", 81, 1560, 128)]


def list_checksum(row_ptr, col_idx):
    rows = np.repeat(np.arange(row_ptr.size - 1, dtype=np.uint64), np.diff(row_ptr).astype(np.int64))
    pos = np.arange(col_idx.size, dtype=np.uint64)
    x = (rows * np.uint64(1000003) + col_idx.astype(np.uint64) * np.uint64(7919) + pos * np.uint64(31) + np.uint64(1))
    x = (x * np.uint64(0x9E3779B97F4A7C15)) >> np.uint64(3)
    return int(np.bitwise_xor.reduce(x)) if x.size else 0


def main():
    lines = ["# workload sink nnz min_row max_row checksum visible_token_pairs   (written by make_block_counts.py from oracle/mask_scan.c)"]
    for name, f, s, block in SHAPES:
        for sink in (0, 1):
            t = time.time()
            nb = -(-f * s // block)
            total = 0
            ptr_parts, idx_parts = [np.zeros(1, dtype=np.int64)], []
            for a in range(0, nb, 256):                       # scan in slabs to bound memory
                bitmap, cnt = obuild.mask_scan(f, s, block, sink, a, min(nb, a + 256))
                total += cnt
                p, i = om.block_lists(bitmap)
                ptr_parts.append(p[1:].astype(np.int64) + ptr_parts[-1][-1])
                idx_parts.append(i)
            row_ptr = np.concatenate(ptr_parts)
            col_idx = np.concatenate(idx_parts)
            lens = np.diff(row_ptr)
            lines.append(f"{name} {sink} {int(row_ptr[-1])} {int(lens.min())} {int(lens.max())} {list_checksum(row_ptr, col_idx)} {total}")
            print(lines[-1], f"({time.time() - t:.1f}s)", flush=True)
    with open(os.path.join(ROOT, "tests", "golden", "block_counts.txt"), "w") as fh:
        fh.write("\n".join(lines) + "\n")


if __name__ == "__main__":
    main()
