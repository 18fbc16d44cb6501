"""Writes tests/golden/abi_forward_fixture.txt: expected block lists and forward rows for the
plain-C program tests/abi_gpu/abi_forward.c, computed by the oracle alone.

Inputs: 8-bit integers / 64 from a 64-bit linear congruential generator (exact in bf16), the
same recipe the C program repeats; they carry none of the method's arithmetic.

    python tests/golden/make_abi_fixture.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import attention as oa   # noqa: E402
from oracle import mask as om        # noqa: E402

F, S, BLOCK, D, B, H, SINK = 12, 320, 64, 64, 1, 2, 1
SEED = 0x5241444941
ROWS = (0, 63, 64, 1000, 1919, 2500, 3333, 3839)
MASK64 = (1 << 64) - 1


def lcg_values(seed, count):
    """count values in {-128..127}/64 from state' = state * 6364136223846793005 + 1442695040888963407."""
    out = np.empty(count, dtype=np.float64)
    state = seed & MASK64
    for i in range(count):
        state = (state * 6364136223846793005 + 1442695040888963407) & MASK64
        out[i] = (((state >> 40) & 0xFF) - 128) / 64.0
    return out


def main():
    n = F * S
    q, k, v = (lcg_values(SEED + t, B * H * n * D).reshape(B, H, n, D) for t in (1, 2, 3))
    scale = 1.0 / np.sqrt(D)
    bitmap = om.block_mask(F, S, BLOCK, SINK)
    row_ptr, col_idx = om.block_lists(bitmap)
    lines = ["# expected values for tests/abi_gpu/abi_forward.c, written by tests/golden/make_abi_fixture.py (oracle only)",
             "# Sec. 4.2 mask (sink of App. A.1) reduced to blocks, then Eq. 2 on the listed blocks; float64",
             f"shape {F} {S} {BLOCK} {D} {B} {H} {SINK}", f"seed {SEED}", f"nnz {int(row_ptr[-1])}",
             "row_ptr " + " ".join(str(int(t)) for t in row_ptr), "col_idx " + " ".join(str(int(t)) for t in col_idx),
             f"rows {len(ROWS) * B * H}"]
    for b in range(B):
        for h in range(H):
            for r in ROWS:
                keys = np.flatnonzero(om.expand_block_row(bitmap[r // BLOCK], BLOCK, n))
                o, lse, _ = oa.attention_rows_keyset(q[b, h, r:r + 1], k[b, h], v[b, h], keys, scale)
                lines.append(f"{b} {h} {r} {lse[0]:.9e} " + " ".join(f"{t:.9e}" for t in o[0]))
    path = os.path.join(ROOT, "tests", "golden", "abi_forward_fixture.txt")
    open(path, "w").write("\n".join(lines) + "\n")
    print(path, os.path.getsize(path), "bytes")


if __name__ == "__main__":
    main()
