"""Pins of the mask oracle against what the paper and arithmetic fix (CPU only)."""
import itertools
from fractions import Fraction
import math
import os

import numpy as np
import pytest

from oracle import build as obuild
from oracle import mask as om


def _facts(golden_dir):
    out = {}
    for line in open(os.path.join(golden_dir, "paper_facts.txt")):
        line = line.split("#")[0].split()
        if len(line) == 2:
            out[line[0]] = int(line[1])
    return out


SHAPES = [(1, 1), (1, 5), (2, 3), (3, 4), (5, 1), (6, 2), (7, 8), (12, 6), (16, 3), (17, 5), (40, 2), (33, 7), (9, 16)]


# ---- structure the paper states -------------------------------------------------------------

@pytest.mark.parametrize("f,s", SHAPES)
def test_central_band_and_sink_are_dense(f, s):
    # App. A.1, mask M^(1): every pair with |i-j| <= 1 or j = 0 is kept.
    m = om.token_mask_4d(f, s, sink_frames=1)
    for i in range(f):
        for j in range(f):
            if abs(i - j) <= 1 or j == 0:
                assert m[i, j].all(), (i, j)


def test_band_count_matches_figure(golden_dir):
    # Sec. 4.2: 2*ceil(log2(max(f,2))) - 1 bands; Fig. 4(a): f = 12 -> 7.
    facts = _facts(golden_dir)
    for f in range(1, 70):
        bands = {om.band_index(i, j) for i in range(f) for j in range(f)}
        assert len(bands) == 2 * math.ceil(math.log2(max(f, 2))) - 1, f
        assert bands == set(range(-max(bands), max(bands) + 1))
    assert len({om.band_index(i, j) for i in range(12) for j in range(12)}) == facts["bands_f12"]


def test_band_widths_double_except_band_one(golden_dir):
    # Fig. 4(a) caption: each band doubles the width of its predecessor, except band +-1.
    facts = _facts(golden_dir)
    f = 200
    width = {}
    for j in range(f):
        r = om.band_index(0, j)
        width[r] = width.get(r, 0) + 1
    # band 0 holds d = 0, 1 on this side (d = -1, 0, 1 in total)
    assert 2 * width[0] - 1 == facts["band0_frames"]
    assert width[1] == 2
    for r in range(2, 7):
        assert width[r] == 2 * width[r - 1]


@pytest.mark.parametrize("f,s", [(12, 16), (20, 24), (33, 40), (9, 7)])
def test_diagonal_width_interior_rows(f, s):
    # Sec. 4.2: diagonal width floor(s / 2^floor(log2 max(|i-j|,1))); when it is >= 1 an interior
    # query position keeps 2*width - 1 keys of that frame, and the density halves per band.
    m = om.token_mask_4d(f, s, sink_frames=0)
    for i in range(f):
        for j in range(f):
            d = abs(i - j)
            w = s // om.pow2_floor(d)
            if w < 1:
                continue
            counts = m[i, j].sum(axis=1)
            for k in range(s):
                if k >= w - 1 and k <= s - w:
                    assert counts[k] == 2 * w - 1
                assert counts[k] == min(s - 1, k + w - 1) - max(0, k - w + 1) + 1
            # kept keys are exactly a band around k = l
            kk, ll = np.nonzero(m[i, j])
            assert (np.abs(kk - ll) <= w - 1).all()


@pytest.mark.parametrize("f,s", SHAPES)
def test_symmetry_without_sink(f, s):
    # The definition depends on |i-j| and |k-l| only => M~[i,j,k,l] = M~[j,i,l,k].
    m = om.token_mask_4d(f, s, sink_frames=0)
    assert (m == m.transpose(1, 0, 3, 2)).all()
    flat = om.flatten_mask(m)
    assert (flat == flat.T).all()


def test_sink_is_column_only():
    m1 = om.token_mask_4d(20, 3, sink_frames=1)
    m0 = om.token_mask_4d(20, 3, sink_frames=0)
    assert m1[:, 0].all()
    assert (m1[:, 1:] == m0[:, 1:]).all()
    m2 = om.token_mask_4d(20, 3, sink_frames=2)
    assert m2[:, :2].all() and (m2[:, 2:] == m0[:, 2:]).all()


def test_width_below_one_worked_example(golden_dir):
    # Sec. 4.2: below width 1 the diagonal is kept only where |i-j| mod ceil(2^r / s) = 0.
    want = {}
    for line in open(os.path.join(golden_dir, "width_lt1_s2_f40.txt")):
        line = line.split("#")[0].split()
        if len(line) == 2:
            want[int(line[0])] = int(line[1])
    f, s = 40, 2
    m = om.token_mask_4d(f, s, sink_frames=0)
    for i in range(f):
        for j in range(f):
            d = abs(i - j)
            assert int(m[i, j].sum()) == want.get(d, 0), (i, j)
            if want.get(d, 0) == 2:
                assert m[i, j, 0, 0] and m[i, j, 1, 1]


def test_subsampled_bands_keep_amortized_density():
    # Sec. 4.2: the sub-sampling keeps "the same amortized attention density decay": a band
    # with 2^r >= s distances (s a power of two) keeps exactly s single diagonals per side.
    for s in (1, 2, 4, 8):
        f = 300
        m = om.token_mask_rows(f, s, 0, rows=[0])[0].reshape(f, s)      # query (0, 0)
        for r in range(int(math.log2(s)), 8):
            kept = sum(bool(m[d].any()) for d in range(2 ** r, 2 ** (r + 1)))
            assert kept == min(s, 2 ** r)


# ---- counts: closed form, bound ---------------------------------------------------------------

def closed_form_visible(f, s, sink_frames):
    """Visible token pairs, counted per frame pair from the geometry (independent of any array):
    a band |k-l| <= w-1 inside an s x s square holds s + 2*sum_{t=1}^{w-1}(s-t) cells."""
    total = 0
    for i in range(f):
        for j in range(f):
            d = abs(i - j)
            b = 1
            while 2 * b <= max(d, 1):
                b *= 2
            if j < sink_frames:
                total += s * s
            elif b <= s:
                w = s // b
                total += s + 2 * (w - 1) * s - (w - 1) * w
            elif d % ((b + s - 1) // s) == 0:
                total += s
    return total


@pytest.mark.parametrize("f,s", SHAPES + [(64, 5), (100, 3), (50, 12)])
@pytest.mark.parametrize("sink", [0, 1, 3])
def test_visible_count_closed_form_small(f, s, sink):
    m = om.token_mask_4d(f, s, sink_frames=sink)
    assert int(m.sum()) == closed_form_visible(f, s, sink)
    _, total = obuild.mask_scan(f, s, 4, sink)
    assert total == closed_form_visible(f, s, sink)


@pytest.mark.parametrize("f,s,block", [(8, 256, 64), (21, 1560, 128)])
def test_visible_count_closed_form_workloads(f, s, block):
    for sink in (0, 1):
        _, total = obuild.mask_scan(f, s, block, sink)
        assert total == closed_form_visible(f, s, sink)


def test_complexity_bound():
    # Eq. 4-5 / App. A.1: #zeros <= 4 s^2 f log2 f  (= 4 s n (log2 n - log2 s)), f >= 2.
    for f in list(range(2, 40)) + [64, 100, 129, 199]:
        for s in (1, 2, 3, 5, 8, 12, 64, 256, 1560, 3600):
            for sink in (0, 1):
                assert closed_form_visible(f, s, sink) <= 4 * s * s * f * math.log2(f) + 1e-9, (f, s, sink)


def test_n_log_n_growth():
    # Eq. 5: at fixed s the cost grows as n log n: visible keys per query <= 4 s log2 f, and
    # doubling f adds at most a constant (4 s) per query instead of doubling it.
    s = 16
    per_row = {}
    for f in (8, 16, 32, 64, 128, 256):
        per_row[f] = closed_form_visible(f, s, 1) / (f * s)
        assert per_row[f] <= 4 * s * math.log2(f)
    for f in (8, 16, 32, 64, 128):
        assert per_row[2 * f] - per_row[f] <= 4 * s
        assert per_row[2 * f] < 1.6 * per_row[f]
    # dense attention would be f*s keys per query
    assert per_row[256] < 0.1 * 256 * s


# ---- three writings of the definition agree; block reduction by brute force ----------------------

@pytest.mark.parametrize("f,s", SHAPES)
@pytest.mark.parametrize("sink", [0, 1, 2])
def test_scalar_numpy_and_c_agree(f, s, sink):
    m = om.token_mask_4d(f, s, sink_frames=sink)
    for i, j, k, l in itertools.product(range(f), range(f), range(s), range(s)):
        assert bool(m[i, j, k, l]) == om.token_visible(f, s, sink, i, j, k, l)
    flat = om.flatten_mask(m)
    assert flat[(f - 1) * s + (s - 1), 0] == m[f - 1, 0, s - 1, 0]
    rows = om.token_mask_rows(f, s, sink, np.arange(f * s))
    assert (rows == flat).all()
    bitmap1, total = obuild.mask_scan(f, s, 1, sink)       # block = 1: the token mask itself
    assert (bitmap1 == flat).all() and total == int(flat.sum())


def brute_block_mask(flat, block):
    n = flat.shape[0]
    nb = -(-n // block)
    bm = np.zeros((nb, nb), dtype=bool)
    for q in range(n):
        for c in range(n):
            if flat[q, c]:
                bm[q // block, c // block] = True
    return bm


@pytest.mark.parametrize("f,s,block", [(6, 5, 4), (7, 8, 3), (12, 6, 8), (40, 2, 8), (5, 12, 5), (3, 3, 16), (9, 16, 16), (17, 5, 7)])
@pytest.mark.parametrize("sink", [0, 1])
def test_block_reduction_brute_force(f, s, block, sink):
    flat = om.flatten_mask(om.token_mask_4d(f, s, sink))
    want = brute_block_mask(flat, block)
    assert (om.block_mask(f, s, block, sink) == want).all()
    got, _ = obuild.mask_scan(f, s, block, sink)
    assert (got == want).all()
    row_ptr, col_idx = om.block_lists(want)
    assert row_ptr[-1] == want.sum() and row_ptr[0] == 0
    for qb in range(want.shape[0]):
        cols = col_idx[row_ptr[qb]:row_ptr[qb + 1]]
        assert (np.diff(cols) > 0).all() and want[qb, cols].all()
        assert qb in cols                              # a block always lists itself (d = 0, k = l)
    tp, ti = om.transpose_lists(row_ptr, col_idx, want.shape[1])
    for kb in range(want.shape[1]):
        assert (np.flatnonzero(want[:, kb]) == ti[tp[kb]:tp[kb + 1]]).all()


def test_numpy_rows_and_c_scan_agree_on_tiny_workload():
    f, s, block = 8, 256, 64
    for sink in (0, 1):
        got, _ = obuild.mask_scan(f, s, block, sink)
        assert (om.block_mask(f, s, block, sink) == got).all()


def test_partial_scan_matches_full_scan():
    f, s, block = 21, 1560, 128
    full, _ = obuild.mask_scan(f, s, block, 1)
    part, _ = obuild.mask_scan(f, s, block, 1, 100, 117)
    assert (full[100:117] == part).all()
    sample = [0, 12, 13, 140, 255]
    assert (om.block_mask(f, s, block, 1, qblocks=sample) == full[sample]).all()


def test_expand_block_row():
    row = np.array([True, False, True])
    assert om.expand_block_row(row, 4, 10).tolist() == [True] * 4 + [False] * 4 + [True] * 2


# ---- sparsity knob (width scale c = num/den on frame pairs at distance >= 2) --------------------
# The paper only says the sparsity is adjusted; these pins fix the reading the oracle takes.

SCALES = [(1, 1), (1, 2), (2, 3), (13, 20), (3, 2), (1, 7), (5, 1)]


@pytest.mark.parametrize("f,s", [(7, 8), (12, 6), (17, 5), (9, 16), (40, 2)])
def test_width_scale_of_one_is_the_printed_definition(f, s):
    base = om.token_mask_4d(f, s, 1)
    assert np.array_equal(om.token_mask_4d(f, s, 1, 1, 1), base)
    assert np.array_equal(om.token_mask_4d(f, s, 1, 3, 3), base)          # only the ratio matters
    assert np.array_equal(om.token_mask_4d(f, s, 1, 2, 4), om.token_mask_4d(f, s, 1, 1, 2))


@pytest.mark.parametrize("num,den", SCALES)
def test_width_scale_leaves_near_frames_and_sink_alone(num, den):
    f, s = 12, 10
    m = om.token_mask_4d(f, s, 1, num, den)
    ref = om.token_mask_4d(f, s, 1)
    for i in range(f):
        for j in range(f):
            if abs(i - j) <= 1 or j == 0:
                assert np.array_equal(m[i, j], ref[i, j])
                assert m[i, j].all()


@pytest.mark.parametrize("num,den", SCALES)
@pytest.mark.parametrize("f,s", [(20, 24), (33, 40), (12, 16), (9, 7)])
def test_width_scale_diagonal_width_and_count(f, s, num, den):
    # frame pair at distance d >= 2, band r = floor(log2 d): diagonal of width w = floor(c*s/2^r)
    # (clipped to the frame), i.e. s*(2w-1) - w*(w-1) visible pairs; once w < 1, a single
    # diagonal every ceil(2^r/(c*s)) frames.
    m = om.token_mask_4d(f, s, 0, num, den)
    for i in range(f):
        for j in range(f):
            d = abs(i - j)
            if d < 2:
                continue
            r = int(math.floor(math.log2(d)))
            w = (s * num) // (den * 2 ** r)
            if w >= 1:
                w = min(w, s)
                assert int(m[i, j].sum()) == s * (2 * w - 1) - w * (w - 1), (i, j)
                k = s // 2
                row = np.flatnonzero(m[i, j, k])
                assert row.min() == max(0, k - (w - 1)) and row.max() == min(s - 1, k + w - 1)
            else:
                stride = math.ceil(Fraction(2 ** r * den, s * num))
                want = np.eye(s, dtype=bool) if d % stride == 0 else np.zeros((s, s), dtype=bool)
                assert np.array_equal(m[i, j], want), (i, j)


def test_width_scale_worked_example():
    # f = 4, s = 2, c = 1/2, no sink, derived by hand: distances 0 and 1 are untouched (all four
    # pairs); distance 2 has width floor(0.5*2/2) = 0 < 1 -> stride ceil(2/(0.5*2)) = 2, 2 % 2 = 0:
    # the diagonal stays; distance 3 is in the same band (2^r = 2), 3 % 2 != 0: nothing.
    m = om.flatten_mask(om.token_mask_4d(4, 2, 0, 1, 2)).astype(int)
    full, diag, none = np.ones((2, 2), int), np.eye(2, dtype=int), np.zeros((2, 2), int)
    want = np.block([[full, full, diag, none],
                     [full, full, full, diag],
                     [diag, full, full, full],
                     [none, diag, full, full]])
    assert np.array_equal(m, want)


@pytest.mark.parametrize("num,den", SCALES)
@pytest.mark.parametrize("f,s,block,sink", [(7, 8, 3, 1), (12, 6, 8, 0), (40, 2, 8, 1), (17, 5, 7, 1), (9, 16, 16, 0)])
def test_width_scale_scalar_numpy_and_c_agree(f, s, block, sink, num, den):
    n = f * s
    brute = np.zeros((n, n), dtype=bool)
    for i, j, k, l in itertools.product(range(f), range(f), range(s), range(s)):
        brute[i * s + k, j * s + l] = om.token_visible(f, s, sink, i, j, k, l, num, den)
    rows = om.token_mask_rows(f, s, sink, np.arange(n), num, den)
    assert np.array_equal(rows, brute)
    nb = -(-n // block)
    want = np.zeros((nb, nb), dtype=bool)
    for q, c in zip(*np.nonzero(brute)):
        want[q // block, c // block] = True
    got, total = obuild.mask_scan(f, s, block, sink, 0, None, num, den)
    assert np.array_equal(got, want) and total == int(brute.sum())
    assert np.array_equal(om.block_mask(f, s, block, sink, None, num, den), want)


@pytest.mark.parametrize("num,den", [(1, 1), (13, 20), (1, 7)])
@pytest.mark.parametrize("f,s,sink", [(7, 8, 1), (40, 2, 0), (17, 5, 2)])
def test_c_token_mask_matches_numpy_rows(f, s, sink, num, den):
    n = f * s
    rng = np.random.default_rng(f * s)
    cols = np.sort(rng.choice(n, size=max(1, n // 2), replace=False))
    want = om.token_mask_rows(f, s, sink, np.arange(3, n - 2), num, den)[:, cols]
    assert np.array_equal(obuild.token_mask(f, s, sink, 3, n - 2, cols, num, den), want)
    assert np.array_equal(om.token_mask_rows_cols(f, s, sink, np.arange(3, n - 2), cols, num, den), want)


# ---- text tokens appended to the video sequence --------------------------------------------------

@pytest.mark.parametrize("f,s,block,sink,extra", [(7, 8, 3, 1, 5), (12, 6, 8, 0, 1), (5, 12, 5, 1, 17), (9, 16, 16, 1, 16)])
def test_text_tokens_see_and_are_seen_by_everyone(f, s, block, sink, extra):
    nv, n = f * s, f * s + extra
    full = om.token_mask_rows_with_text(f, s, sink, np.arange(n), extra)
    assert full.shape == (n, n)
    assert np.array_equal(full[:nv, :nv], om.token_mask_rows(f, s, sink, np.arange(nv)))   # video part unchanged
    assert full[nv:].all() and full[:, nv:].all()
    assert np.array_equal(om.token_mask_rows_with_text(f, s, sink, np.arange(nv), 0), full[:nv, :nv])
    nb = -(-n // block)
    want = np.zeros((nb, nb), dtype=bool)
    for q, c in zip(*np.nonzero(full)):
        want[q // block, c // block] = True
    got, total = obuild.mask_scan(f, s, block, sink, 0, None, 1, 1, extra)
    assert np.array_equal(got, want) and total == int(full.sum())
