"""Compiles oracle/mask_scan.c with gcc and loads it through ctypes (test infrastructure)."""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mask_scan.c")
_LIB = os.path.join(_HERE, "liboracle_mask_scan.so")
_handle = None


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC])
    return _LIB


def _lib():
    global _handle
    if _handle is None:
        _handle = ctypes.CDLL(build())
        _handle.radial_mask_scan.restype = ctypes.c_int64
        _handle.radial_mask_scan.argtypes = [ctypes.c_int32] * 9 + [ctypes.c_void_p]
        _handle.radial_token_mask.restype = None
        _handle.radial_token_mask.argtypes = [ctypes.c_int32] * 5 + [ctypes.c_int64] * 3 + [ctypes.c_void_p] * 2
    return _handle


def mask_scan(f: int, s: int, block: int, sink_frames: int, qb_begin: int = 0, qb_end: int | None = None,
              width_num: int = 1, width_den: int = 1, extra_tokens: int = 0):
    """Brute-force block bitmap of query blocks [qb_begin, qb_end) and the visible-token-pair count."""
    n = f * s + extra_tokens
    nb = -(-n // block)
    if qb_end is None:
        qb_end = nb
    bitmap = np.zeros((qb_end - qb_begin, nb), dtype=np.uint8)
    total = _lib().radial_mask_scan(f, s, block, sink_frames, width_num, width_den, extra_tokens, qb_begin, qb_end,
                                    bitmap.ctypes.data)
    return bitmap.astype(bool), int(total)


def token_mask(f: int, s: int, sink_frames: int, q_begin: int, q_end: int, cols, width_num: int = 1, width_den: int = 1):
    """Token mask entries M[q_begin:q_end, cols] by the C loop (same predicate as mask_scan): bool."""
    cols = np.ascontiguousarray(cols, dtype=np.int64)
    out = np.zeros((q_end - q_begin, cols.size), dtype=np.uint8)
    _lib().radial_token_mask(f, s, sink_frames, width_num, width_den, q_begin, q_end, cols.size,
                             cols.ctypes.data, out.ctypes.data)
    return out.astype(bool)
