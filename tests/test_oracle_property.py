"""Randomised cross-checks of the mask oracle's three forms (scalar definition, numpy, C scan)
and of invariants the paper states, on small random geometries (CPU only)."""
import numpy as np
from hypothesis import given, settings, strategies as st

from oracle import build as obuild
from oracle import mask as om

geometry = st.tuples(st.integers(1, 24), st.integers(1, 14), st.sampled_from([2, 3, 4, 5, 8, 16]), st.integers(0, 3),
                     st.integers(1, 9), st.integers(1, 9), st.integers(0, 9))


@settings(max_examples=60, deadline=None)
@given(geometry)
def test_three_forms_agree(geo):
    f, s, block, sink, num, den, extra = geo
    nv, n = f * s, f * s + extra
    brute = np.ones((n, n), dtype=bool)
    for q in range(nv):
        for c in range(nv):
            brute[q, c] = om.token_visible(f, s, sink, q // s, c // s, q % s, c % s, num, den)
    rows = om.token_mask_rows_with_text(f, s, sink, np.arange(n), extra, num, den)
    assert np.array_equal(rows, brute)
    if extra == 0:
        assert np.array_equal(obuild.token_mask(f, s, sink, 0, n, np.arange(n), num, den), brute)
    nb = -(-n // block)
    want = np.zeros((nb, nb), dtype=bool)
    for q, c in zip(*np.nonzero(brute)):
        want[q // block, c // block] = True
    got, total = obuild.mask_scan(f, s, block, sink, 0, None, num, den, extra)
    assert np.array_equal(got, want) and total == int(brute.sum())
    ptr, idx = om.block_lists(got)
    tptr, tidx = om.transpose_lists(ptr, idx, nb)
    assert np.array_equal(om.block_lists(np.ascontiguousarray(got.T))[1], tidx) and tptr[-1] == ptr[-1]


@settings(max_examples=60, deadline=None)
@given(st.integers(1, 40), st.integers(1, 20), st.integers(1, 9), st.integers(1, 9))
def test_invariants(f, s, num, den):
    m = om.token_mask_4d(f, s, 0, num, den)
    # symmetric in the temporal distance and in space (no sink)
    assert np.array_equal(m, m.transpose(1, 0, 2, 3)) and np.array_equal(m, m.transpose(0, 1, 3, 2))
    # every token sees itself, its own frame and the neighbouring frames completely
    for i in range(f):
        for j in range(max(0, i - 1), min(f, i + 2)):
            assert m[i, j].all()
    # the visible pairs of a frame pair depend on the distance only
    for d in range(f):
        ref = m[0, d]
        for i in range(1, f - d):
            assert np.array_equal(m[i, i + d], ref)
    if num == den:                                       # the printed mask: bound of the complexity analysis (f >= 2)
        assert f < 2 or int(m.sum()) <= 4 * s * s * f * max(1.0, np.log2(f))
