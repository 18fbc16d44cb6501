"""GPU mask builder vs the brute-force oracle: bit-exact lists (run with -m gpu)."""
import os

import numpy as np
import pytest

from oracle import build as obuild
from oracle import mask as om
from paper_2506_19852_amd import binding as rb
from paper_2506_19852_amd.workloads import WORKLOADS

pytestmark = pytest.mark.gpu

SMALL = [
    # f, s, block
    (300, 2, 64), (300, 2, 128), (100, 7, 64), (33, 40, 64), (33, 40, 128), (16, 100, 64), (5, 1000, 128),
    (1, 500, 64), (2, 64, 64), (64, 24, 128), (129, 1, 64), (700, 3, 128), (8, 256, 64), (3, 129, 128), (1, 1, 64),
    (1024, 1, 128), (40, 130, 64),
]


def _lists_from_bitmap(bitmap):
    return om.block_lists(bitmap)


@pytest.mark.parametrize("f,s,block", SMALL)
@pytest.mark.parametrize("sink", [0, 1, 2])
def test_small_shapes_bit_exact(f, s, block, sink):
    print(f"mask f={f} s={s} block={block} sink={sink}", flush=True)
    bitmap, _ = obuild.mask_scan(f, s, block, sink)
    want_ptr, want_idx = _lists_from_bitmap(bitmap)
    m = rb.radial_mask_build(f, s, block, sink, rb.RADIAL_MASK_TRANSPOSE)
    info = rb.radial_mask_info(m)
    assert info == {"n_tokens": f * s, "block": block, "n_blocks": bitmap.shape[0], "nnz": int(bitmap.sum()),
                    "flags": rb.RADIAL_MASK_TRANSPOSE}
    got_ptr, got_idx = rb.radial_mask_copy_to_host(m)
    assert np.array_equal(got_ptr, want_ptr) and np.array_equal(got_idx, want_idx)
    t_ptr, t_idx = rb.radial_mask_copy_transpose_to_host(m)
    wt_ptr, wt_idx = _lists_from_bitmap(np.ascontiguousarray(bitmap.T))
    assert np.array_equal(t_ptr, wt_ptr) and np.array_equal(t_idx, wt_idx)
    m.free()


def _golden_counts(golden_dir):
    out = {}
    for line in open(os.path.join(golden_dir, "block_counts.txt")):
        line = line.split("#")[0].split()
        if len(line) == 7:
            out[(line[0], int(line[1]))] = tuple(int(x) for x in line[2:])
    return out


def list_checksum(row_ptr, col_idx):
    """Order-sensitive 61-bit checksum of a compressed list (same formula as the golden writer)."""
    rows = np.repeat(np.arange(row_ptr.size - 1, dtype=np.uint64), np.diff(row_ptr).astype(np.int64))
    pos = np.arange(col_idx.size, dtype=np.uint64)
    x = (rows * np.uint64(1000003) + col_idx.astype(np.uint64) * np.uint64(7919) + pos * np.uint64(31) + np.uint64(1))
    x = (x * np.uint64(0x9E3779B97F4A7C15)) >> np.uint64(3)
    return int(np.bitwise_xor.reduce(x)) if x.size else 0


@pytest.mark.parametrize("name", list(WORKLOADS))
@pytest.mark.parametrize("sink", [0, 1])
def test_workload_masks(name, sink, golden_dir):
    w = WORKLOADS[name]
    f, s, block = w.frames, w.tokens_per_frame, w.block
    print(f"mask workload {name} sink={sink}", flush=True)
    m = rb.radial_mask_build(f, s, block, sink, rb.RADIAL_MASK_TRANSPOSE)
    got_ptr, got_idx = rb.radial_mask_copy_to_host(m)
    nb = got_ptr.size - 1
    lens = np.diff(got_ptr)
    # whole list against the numbers the oracle's full brute-force scan wrote down
    nnz, lmin, lmax, csum, _ = _golden_counts(golden_dir)[(name, sink)]
    assert (int(got_ptr[-1]), int(lens.min()), int(lens.max())) == (nnz, lmin, lmax)
    assert list_checksum(got_ptr, got_idx) == csum
    # and a live brute-force scan: everything for the smaller workloads, sampled query blocks for the rest
    if w.N <= 40000:
        ranges = [(0, nb)]
    else:
        starts = sorted({0, nb - 8, nb // 2, nb // 3, (s // block) - 1, (5 * s) // block, nb - 40})
        ranges = [(a, min(nb, a + 8)) for a in starts if a >= 0]
    for a, b in ranges:
        bitmap, _ = obuild.mask_scan(f, s, block, sink, a, b)
        for qb in range(a, b):
            assert np.array_equal(got_idx[got_ptr[qb]:got_ptr[qb + 1]], np.flatnonzero(bitmap[qb - a])), (name, qb)
    # transpose is consistent with the list itself
    t_ptr, t_idx = rb.radial_mask_copy_transpose_to_host(m)
    rows = np.repeat(np.arange(nb), lens)
    order = np.lexsort((rows, got_idx))
    assert np.array_equal(t_idx, rows[order].astype(np.int32))
    assert np.array_equal(np.diff(t_ptr), np.bincount(got_idx, minlength=nb))
    m.free()


def test_dense_and_user_lists():
    m = rb.radial_mask_build_dense(1000, 128, rb.RADIAL_MASK_TRANSPOSE)
    ptr, idx = rb.radial_mask_copy_to_host(m)
    assert np.array_equal(ptr, np.arange(9) * 8) and np.array_equal(idx, np.tile(np.arange(8), 8))
    tp, ti = rb.radial_mask_copy_transpose_to_host(m)
    assert np.array_equal(tp, ptr) and np.array_equal(ti, idx)
    m.free()
    row_ptr = np.array([0, 2, 2, 3, 6], dtype=np.int32)
    col_idx = np.array([0, 3, 1, 0, 1, 2], dtype=np.int32)
    m = rb.radial_mask_from_csr(4 * 64 - 5, 64, row_ptr, col_idx, rb.RADIAL_MASK_TRANSPOSE)
    p2, i2 = rb.radial_mask_copy_to_host(m)
    assert np.array_equal(p2, row_ptr) and np.array_equal(i2, col_idx)
    tp, ti = rb.radial_mask_copy_transpose_to_host(m)
    assert np.array_equal(tp, [0, 2, 4, 5, 6]) and np.array_equal(ti, [0, 3, 2, 3, 3, 0])
    m.free()
    with pytest.raises(rb.RadialError) as e:
        rb.radial_mask_from_csr(256, 64, np.array([0, 2, 2, 2, 2]), np.array([1, 1]))
    assert e.value.code == -1
    with pytest.raises(rb.RadialError):
        rb.radial_mask_from_csr(256, 64, np.array([0, 1, 1, 1, 1]), np.array([4]))
    with pytest.raises(rb.RadialError):
        rb.radial_mask_copy_transpose_to_host(rb.radial_mask_build(4, 64, 64, 1, 0))
