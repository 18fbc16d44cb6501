"""Radial mask, written out from its definition (test oracle; see oracle/__init__.py).

Notation follows the paper: f frames, s tokens per frame, n = f*s tokens; query token
(i, k) = frame i, spatial position k; key token (j, l).  ``True`` means "may attend"
(the paper's 0 entry), ``False`` means suppressed (the paper's -inf entry).

Readings taken where the paper leaves a choice (each is also listed in the design notes):

* floor(log2(.)) and ceil(./s) are evaluated in integers (bit length, ceiling division);
  the real-valued comparison |k-l|+1 <= s/2^r is the integer comparison (|k-l|+1)*2^r <= s.
* The attention sink (Sec. 4.2 last paragraph of the formal definition; App. A.1 mask
  M^(1): "or j = 0") is OR-ed onto the equation: key frames j < sink_frames are visible
  to every query.
* Block reduction (Sec. 4.2, "Hardware-friendly block sparsity" gives only the block size):
  blocks tile the flattened token index from 0; a (query block, key block) pair is listed
  iff ANY token pair inside it is visible; a listed block is computed densely, so the
  function the library evaluates is Eq. 2 under the block-expanded mask.
* Sparsity knob (App. D / Sec. 5.1 say the mask's sparsity is "adjusted" to a compute budget
  without defining how): a rational width scale c = width_num / width_den applied to frame
  pairs at distance >= 2 only.  There the diagonal width floor(s / 2^r) becomes
  floor(c * s / 2^r), i.e. (|k-l|+1) * 2^r * width_den <= s * width_num, and once that width
  drops below 1 the diagonal is kept every ceil(2^r / (c * s)) frames.  c = 1 is the printed
  definition; frame pairs at distance 0 and 1 and the sink are never scaled.
* Text tokens (the video models the paper evaluates append prompt tokens to the video
  sequence, Sec. 5.1; the paper does not say how the mask treats them): ``extra_tokens``
  tokens after the f*s video tokens attend to every token and are attended by every token.
"""
from __future__ import annotations

import numpy as np


def pow2_floor(d: int) -> int:
    """2^floor(log2(max(d, 1))) -- the temporal band base of Sec. 4.2."""
    d = max(int(d), 1)
    return 1 << (d.bit_length() - 1)


def band_index(i: int, j: int) -> int:
    """sign(j - i) * floor(log2(max(|i - j|, 1)))  (Sec. 4.2, temporal density decay)."""
    d = abs(i - j)
    r = max(d, 1).bit_length() - 1
    return r if j > i else (-r if j < i else 0)


def token_visible(f: int, s: int, sink_frames: int, i: int, j: int, k: int, l: int,
                  width_num: int = 1, width_den: int = 1) -> bool:
    """One entry of the 4-D mask of Sec. 4.2 (formal definition) OR the sink of App. A.1."""
    assert 0 <= i < f and 0 <= j < f and 0 <= k < s and 0 <= l < s
    assert width_num >= 1 and width_den >= 1
    if j < sink_frames:                                  # attention sink
        return True
    d = abs(i - j)
    b = pow2_floor(d)
    num, den = (width_num, width_den) if d >= 2 else (1, 1)   # the knob leaves d = 0, 1 alone
    if b * den <= s * num and (abs(k - l) + 1) * b * den <= s * num:   # case 1: width floor(c*s/b)
        return True
    stride = -(-(b * den) // (s * num))                  # ceil(b / (c*s))
    if d % stride == 0 and k == l:                       # case 2: sub-sampled single diagonals
        return True
    return False


def token_mask_4d(f: int, s: int, sink_frames: int = 1, width_num: int = 1, width_den: int = 1) -> np.ndarray:
    """The whole mask M~[i, j, k, l] as a bool array (small f*s only)."""
    i = np.arange(f, dtype=np.int64)[:, None, None, None]
    j = np.arange(f, dtype=np.int64)[None, :, None, None]
    k = np.arange(s, dtype=np.int64)[None, None, :, None]
    l = np.arange(s, dtype=np.int64)[None, None, None, :]
    return _visible_arrays(s, sink_frames, i, j, k, l, width_num, width_den)


def _visible_arrays(s, sink_frames, i, j, k, l, width_num=1, width_den=1):
    d = np.abs(i - j)
    dm = np.maximum(d, 1)
    # floor(log2(dm)) via exact integer search (no floating point anywhere in the mask)
    r = np.zeros_like(dm)
    t = dm.copy()
    while np.any(t > 1):
        r = r + (t > 1)
        t = t >> 1
    b = np.int64(1) << r
    num = np.where(d >= 2, np.int64(width_num), np.int64(1))
    den = np.where(d >= 2, np.int64(width_den), np.int64(1))
    case1 = (b * den <= s * num) & ((np.abs(k - l) + 1) * b * den <= s * num)
    stride = (b * den + s * num - 1) // (s * num)
    case2 = ((d % stride) == 0) & (k == l)
    sink = j < sink_frames
    return case1 | case2 | sink


def flatten_mask(m4: np.ndarray) -> np.ndarray:
    """M[i*s + k, j*s + l] = M~[i, j, k, l]  (Sec. 4.2, after the formal definition)."""
    f, f2, s, s2 = m4.shape
    assert f == f2 and s == s2
    return np.ascontiguousarray(m4.transpose(0, 2, 1, 3)).reshape(f * s, f * s)


def token_mask_rows(f: int, s: int, sink_frames: int, rows, width_num: int = 1, width_den: int = 1) -> np.ndarray:
    """Rows ``rows`` of the flattened token mask M, bool [len(rows), n]."""
    rows = np.asarray(rows, dtype=np.int64)
    n = f * s
    cols = np.arange(n, dtype=np.int64)
    i = (rows // s)[:, None]
    k = (rows % s)[:, None]
    j = (cols // s)[None, :]
    l = (cols % s)[None, :]
    return _visible_arrays(s, sink_frames, i, j, k, l, width_num, width_den)


def token_mask_rows_cols(f: int, s: int, sink_frames: int, rows, cols, width_num: int = 1, width_den: int = 1) -> np.ndarray:
    """Entries M[rows, cols] of the flattened token mask, bool [len(rows), len(cols)]."""
    rows = np.asarray(rows, dtype=np.int64)
    cols = np.asarray(cols, dtype=np.int64)
    i = (rows // s)[:, None]
    k = (rows % s)[:, None]
    j = (cols // s)[None, :]
    l = (cols % s)[None, :]
    return _visible_arrays(s, sink_frames, i, j, k, l, width_num, width_den)


def block_any(mask_rows: np.ndarray, block: int) -> np.ndarray:
    """OR-reduce the key axis of token-mask rows into key blocks: bool [rows, ceil(n/block)]."""
    r, n = mask_rows.shape
    nkb = -(-n // block)
    pad = nkb * block - n
    m = np.pad(mask_rows, ((0, 0), (0, pad)), constant_values=False)
    return m.reshape(r, nkb, block).any(axis=2)


def block_mask(f: int, s: int, block: int, sink_frames: int = 1, qblocks=None,
               width_num: int = 1, width_den: int = 1) -> np.ndarray:
    """Block bitmap [len(qblocks), nkb]: entry true iff any token pair of the block pair is visible."""
    n = f * s
    nqb = -(-n // block)
    if qblocks is None:
        qblocks = range(nqb)
    out = []
    for qb in qblocks:
        rows = np.arange(qb * block, min(n, (qb + 1) * block))
        out.append(block_any(token_mask_rows(f, s, sink_frames, rows, width_num, width_den), block).any(axis=0))
    return np.array(out, dtype=bool).reshape(len(out), -(-n // block))


def block_lists(bitmap: np.ndarray):
    """Compressed form of a block bitmap: row_ptr [nqb+1], col_idx [nnz] (ascending per row)."""
    nqb = bitmap.shape[0]
    row_ptr = np.zeros(nqb + 1, dtype=np.int32)
    cols = []
    for qb in range(nqb):
        c = np.flatnonzero(bitmap[qb]).astype(np.int32)
        cols.append(c)
        row_ptr[qb + 1] = row_ptr[qb] + c.size
    col_idx = np.concatenate(cols) if cols else np.zeros(0, dtype=np.int32)
    return row_ptr, col_idx.astype(np.int32)


def transpose_lists(row_ptr: np.ndarray, col_idx: np.ndarray, nkb: int):
    """Per key block, the ascending list of query blocks that list it."""
    nqb = row_ptr.size - 1
    bm = np.zeros((nqb, nkb), dtype=bool)
    for qb in range(nqb):
        bm[qb, col_idx[row_ptr[qb]:row_ptr[qb + 1]]] = True
    return block_lists(np.ascontiguousarray(bm.T))


def expand_block_row(block_row: np.ndarray, block: int, n: int) -> np.ndarray:
    """Token-level visibility of one query block under block-dense semantics: bool [n]."""
    return np.repeat(block_row, block)[:n]


def token_mask_rows_with_text(f: int, s: int, sink_frames: int, rows, extra_tokens: int,
                              width_num: int = 1, width_den: int = 1) -> np.ndarray:
    """Rows of the token mask of a sequence of f*s video tokens followed by extra_tokens text
    tokens: bool [len(rows), f*s + extra_tokens]."""
    rows = np.asarray(rows, dtype=np.int64)
    nv = f * s
    out = np.ones((rows.size, nv + extra_tokens), dtype=bool)          # text rows and text columns
    video = rows < nv
    if video.any():
        out[np.flatnonzero(video), :nv] = token_mask_rows(f, s, sink_frames, rows[video], width_num, width_den)
    return out
