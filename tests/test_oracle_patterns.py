"""Pins of the oracle's other static masks (CPU only)."""
import itertools

import numpy as np
import pytest

from oracle import mask as om
from oracle import patterns as op


@pytest.mark.parametrize("f,s,sink", [(6, 8, 1), (12, 16, 0), (8, 5, 2), (3, 40, 1)])
def test_radial_mask_is_banded_while_widths_are_at_least_one(f, s, sink):
    # an independent route to the same mask: the formal definition vs the banded rule with the
    # radial width table
    hw = op.half_widths_radial(f, s)
    rows = np.arange(f * s)
    assert np.array_equal(op.banded_mask_rows(f, s, sink, hw, rows), om.token_mask_rows(f, s, sink, rows))


def test_radial_width_table_refuses_subsampled_regime():
    with pytest.raises(AssertionError):
        op.half_widths_radial(40, 4)


@pytest.mark.parametrize("f,s", [(7, 6), (10, 9)])
def test_scalar_and_vector_forms_agree(f, s):
    rng = np.random.default_rng(3)
    hw = rng.integers(-1, s + 2, size=f).tolist()
    rows = op.banded_mask_rows(f, s, 1, hw, np.arange(f * s))
    for i, j, k, l in itertools.product(range(f), range(f), range(s), range(s)):
        assert rows[i * s + k, j * s + l] == op.banded_visible(s, 1, hw, i, j, k, l)


def test_spatial_head_counts():
    f, s, w = 9, 7, 2
    m = op.banded_mask_rows(f, s, 0, op.half_widths_spatial(f, s, w), np.arange(f * s))
    # row of frame i sees every token of frames i-w .. i+w
    for i in range(f):
        frames = min(f - 1, i + w) - max(0, i - w) + 1
        assert (m[i * s:(i + 1) * s].sum(axis=1) == frames * s).all()
    assert np.array_equal(m, m.T)


def test_temporal_head_counts():
    f, s, h = 5, 11, 2
    m = op.banded_mask_rows(f, s, 0, op.half_widths_temporal(f, s, h), np.arange(f * s))
    for k in range(s):
        per_frame = min(s - 1, k + h) - max(0, k - h) + 1
        assert (m[k::s].sum(axis=1) == f * per_frame).all()
    # same position in every frame is always visible
    assert all(m[i * s + k, j * s + k] for i in range(f) for j in range(f) for k in range(s))


def test_sliding_window_is_intersection_of_spatial_and_temporal():
    f, s, w, h = 8, 9, 1, 3
    rows = np.arange(f * s)
    a = op.banded_mask_rows(f, s, 0, op.half_widths_spatial(f, s, w), rows)
    b = op.banded_mask_rows(f, s, 0, op.half_widths_temporal(f, s, h), rows)
    c = op.banded_mask_rows(f, s, 0, op.half_widths_sliding(f, s, w, h), rows)
    assert np.array_equal(c, a & b)


def test_harmonic_widths():
    f, s = 30, 24
    hw = op.half_widths_harmonic(f, s)
    assert hw[0] == hw[1] == s - 1
    for d in range(2, f):
        assert hw[d] + 1 == s // d                      # width inversely proportional to d
    assert hw[25] == -1                                 # below one: nothing
    # visible pairs over all frame pairs ~ s^2 * sum_d 1/d: O(n log n) like the radial mask
    m = op.banded_mask_rows(f, s, 0, hw, np.arange(f * s))
    want = 0
    for i in range(f):
        for j in range(f):
            w = hw[abs(i - j)] + 1
            want += s * (2 * w - 1) - w * (w - 1) if w >= 1 else 0
    assert int(m.sum()) == want


def test_power_of_two_rows():
    n = 70
    m = op.power_of_two_rows(n, np.arange(n))
    for q in range(n):
        want = {c for c in range(n) if abs(q - c) in (0, 1, 2, 4, 8, 16, 32, 64)}
        assert set(np.flatnonzero(m[q])) == want
    assert int(op.power_of_two_rows(1 << 12, [0]).sum()) == 13      # 0 and 2^0 .. 2^11
    m2 = op.power_of_two_rows(n, np.arange(n), local=5)
    assert all(m2[q, c] for q in range(n) for c in range(n) if abs(q - c) <= 5)


def test_block_bitmap_brute_force():
    f, s, block = 7, 6, 4
    hw = op.half_widths_harmonic(f, s)
    n = f * s
    full = op.banded_mask_rows(f, s, 1, hw, np.arange(n))
    nb = -(-n // block)
    want = np.zeros((nb, nb), dtype=bool)
    for q, c in zip(*np.nonzero(full)):
        want[q // block, c // block] = True
    got = op.block_bitmap(lambda rows: op.banded_mask_rows(f, s, 1, hw, rows), n, block)
    assert np.array_equal(got, want)
