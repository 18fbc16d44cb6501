"""Other static video-attention masks the paper compares with (test oracle; see oracle/__init__.py).

The paper describes them in a sentence each (Sec. 3 "Spatiotemporal Energy Decay", Sec. 5.1
"Baselines", App. "Comparison with Other O(n log n) Sparsity Patterns") and defines none of
them formally, so every function here states the reading it takes.  Notation as in
oracle/mask.py: query token (i, k), key token (j, l), f frames of s tokens.

Four of the five patterns are *banded*: a key is visible iff it lies in the sink or within a
spatial half width that depends on the frame distance only,

    visible  <=>  j < sink_frames  or  |k - l| <= half_width[|i - j|]      (-1: nothing).

``half_width`` is a plain list of f integers; the generators below fill it.
"""
from __future__ import annotations

import numpy as np


def banded_visible(s: int, sink_frames: int, half_width, i: int, j: int, k: int, l: int) -> bool:
    if j < sink_frames:
        return True
    return abs(k - l) <= half_width[abs(i - j)]


def banded_mask_rows(f: int, s: int, sink_frames: int, half_width, rows) -> np.ndarray:
    """Rows ``rows`` of the flattened token mask of a banded pattern, bool [len(rows), f*s]."""
    hw = np.asarray(half_width, dtype=np.int64)
    assert hw.shape == (f,)
    rows = np.asarray(rows, dtype=np.int64)
    cols = np.arange(f * s, dtype=np.int64)
    i, k = (rows // s)[:, None], (rows % s)[:, None]
    j, l = (cols // s)[None, :], (cols % s)[None, :]
    return (j < sink_frames) | (np.abs(k - l) <= hw[np.abs(i - j)])


def half_widths_spatial(f: int, s: int, frame_window: int):
    """SVG's "spatial head" (Sec. 3: each token attends to nearby tokens within adjacent
    frames).  Reading: every token of the frames at distance <= frame_window, nothing else."""
    return [s - 1 if d <= frame_window else -1 for d in range(f)]


def half_widths_temporal(f: int, s: int, spatial_half_width: int):
    """SVG's "temporal head" (Sec. 3: each token focuses on the same spatial location across
    frames).  Reading: spatial positions within spatial_half_width, in every frame."""
    return [min(spatial_half_width, s - 1)] * f


def half_widths_sliding(f: int, s: int, frame_window: int, spatial_half_width: int):
    """Sliding-window attention local in space and time (Sec. 5.1, STA).  Reading: a window of
    frame_window frames to each side and spatial_half_width positions to each side; the
    spatial position is the flattened one, as everywhere in this code base."""
    return [min(spatial_half_width, s - 1) if d <= frame_window else -1 for d in range(f)]


def half_widths_harmonic(f: int, s: int):
    """Harmonic Series Decay (App., comparison with other O(n log n) patterns): the diagonal
    width is inversely proportional to the distance from the main diagonal.  Reading: width
    floor(s / max(d, 1)) at frame distance d, nothing once that is below one."""
    return [min(s // max(d, 1), s) - 1 for d in range(f)]


def half_widths_radial(f: int, s: int):
    """The radial mask itself as a banded pattern: width floor(s / 2^floor(log2 max(d,1))).
    Only valid while every width is >= 1 (2^floor(log2(f-1)) <= s), because the sub-sampled single
    diagonals of the formal definition are not a function of |i - j| alone."""
    out = []
    for d in range(f):
        b = 1 << (max(d, 1).bit_length() - 1)
        assert b <= s, "the radial mask is banded only while 2^r <= s"
        out.append(s // b - 1)
    return out


def power_of_two_rows(n: int, rows, local: int = 0) -> np.ndarray:
    """PowerAttention (Sec. 5.1: tokens at power-of-two distances).  Reading: on the flattened
    token index, |q - c| is 0, a power of two, or at most ``local``."""
    rows = np.asarray(rows, dtype=np.int64)[:, None]
    cols = np.arange(n, dtype=np.int64)[None, :]
    dist = np.abs(rows - cols)
    return (dist <= local) | ((dist & (dist - 1)) == 0)


def block_bitmap(mask_rows_fn, n: int, block: int) -> np.ndarray:
    """"Any" block cover of a token mask given by a rows -> bool [r, n] function."""
    nb = -(-n // block)
    out = np.zeros((nb, nb), dtype=bool)
    pad = nb * block - n
    for qb in range(nb):
        rows = np.arange(qb * block, min(n, (qb + 1) * block))
        m = np.pad(mask_rows_fn(rows), ((0, 0), (0, pad)), constant_values=False)
        out[qb] = m.reshape(rows.size, nb, block).any(axis=(0, 2))
    return out
