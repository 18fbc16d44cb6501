"""Half-width tables for radial_mask_build_banded: the other static video masks the paper
compares with (Sec. 3, Sec. 5.1 "Baselines", App. on other O(n log n) patterns).

A banded mask lets query token (i, k) attend key token (j, l) iff j is a sink frame or
|k - l| <= half_width[|i - j|]; -1 hides the frame pair.  The paper describes these masks in a
sentence each, so every function states the reading it takes; callers with another reading
pass their own table.

These four functions are caller-side examples, not part of the library: the library's rule is
the table lookup above and nothing else (`bench.py --pattern` uses them to pick example widths).
The tests check the library against the oracle's own definitions of these masks with tables the
test passes in, never against this file.
"""
from __future__ import annotations


def spatial_head(frames: int, tokens_per_frame: int, frame_window: int):
    """Every token of the frames at most frame_window away (the "spatial" head mask)."""
    return [tokens_per_frame - 1 if d <= frame_window else -1 for d in range(frames)]


def temporal_head(frames: int, tokens_per_frame: int, spatial_half_width: int):
    """Positions at most spatial_half_width away, in every frame (the "temporal" head mask)."""
    return [min(spatial_half_width, tokens_per_frame - 1)] * frames


def sliding_window(frames: int, tokens_per_frame: int, frame_window: int, spatial_half_width: int):
    """Local in time and in (flattened) space."""
    hw = min(spatial_half_width, tokens_per_frame - 1)
    return [hw if d <= frame_window else -1 for d in range(frames)]


def harmonic_decay(frames: int, tokens_per_frame: int):
    """Diagonal width floor(s / max(d, 1)): inversely proportional to the frame distance."""
    return [min(tokens_per_frame // max(d, 1), tokens_per_frame) - 1 for d in range(frames)]
