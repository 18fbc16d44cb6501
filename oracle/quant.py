"""8-bit floating-point scores (test oracle; see oracle/__init__.py).

The paper leaves quantisation to other work (Sec. 2 and Sec. 6 call the method orthogonal to
quantised attention kernels) and defines none, so the scheme is this library's own and its
agreement with any published kernel is "parity unpinned".  What is pinned is the number format:
E4M3 of the OCP 8-bit floating point specification (1 sign, 4 exponent bits with bias 7, 3
mantissa bits, subnormals, no infinities, S.1111.111 = NaN, largest finite value 448), written
out here from that definition, and round-to-nearest-even.

Scheme: Q and K are cut into blocks of `block` consecutive tokens of one (batch, head); a block
is stored as E4M3 codes of x / scale with scale = amax / 448 in float32 (1 if the block is all
zero), so the largest magnitude of every block maps to 448.  Scores are
(code values of q) . (code values of k) * scale_q * scale_k; V and everything after the scores
stay as they are.
"""
from __future__ import annotations

import numpy as np

E4M3_MAX = 448.0


def e4m3_decode(codes):
    """Values (float64) of E4M3 codes (uint8); NaN for the two NaN codes."""
    c = np.asarray(codes, dtype=np.uint8).astype(np.int64)
    sign = np.where(c & 0x80, -1.0, 1.0)
    e = (c >> 3) & 0xF
    m = c & 0x7
    normal = np.ldexp(1.0 + m / 8.0, e - 7)
    sub = np.ldexp(m / 8.0, -6)
    val = np.where(e == 0, sub, normal)
    val = np.where((e == 15) & (m == 7), np.nan, val)
    return sign * val


def e4m3_encode(x):
    """E4M3 codes (uint8) of x, round to nearest, ties to the even mantissa.

    |x| must not round above 448 (the quantiser guarantees it); -0.0 keeps its sign.
    """
    x = np.asarray(x, dtype=np.float64)
    a = np.abs(x)
    if np.any(a >= 464.0) or np.any(np.isnan(a)):     # 464 is the midpoint between 448 and the next step
        raise ValueError("value out of the E4M3 range")
    # exponent of the binade, clamped to the subnormal binade; steps of 2^(e-3) inside it
    _, ex = np.frexp(a)                                # a = f * 2^ex, f in [0.5, 1)
    e = np.maximum(ex - 1, -6)
    q = np.rint(np.ldexp(a, 3 - e))                    # multiples of the step, exact; rint = ties to even
    # q in [0, 8) is subnormal (only when e = -6), [8, 16) normal, 16 carries into the next binade
    carry = q >= 16
    e = np.where(carry, e + 1, e)
    q = np.where(carry, 8, q)
    is_sub = q < 8
    code = np.where(is_sub, q, ((e + 7).astype(np.int64) << 3) | (q.astype(np.int64) - 8)).astype(np.int64)
    code = code | np.where(np.signbit(x), 0x80, 0)
    return code.astype(np.uint8)


def quantize_blocks(x, block):
    """x: [n, D] (values representable in float32) -> (codes uint8 [n, D], scales float32 [ceil(n/block)])."""
    x = np.asarray(x, dtype=np.float32)
    n = x.shape[0]
    nb = (n + block - 1) // block
    codes = np.empty(x.shape, dtype=np.uint8)
    scales = np.empty(nb, dtype=np.float32)
    for b in range(nb):
        rows = slice(b * block, min(n, (b + 1) * block))
        amax = np.float32(np.abs(x[rows]).max())
        scale = np.float32(amax / np.float32(E4M3_MAX)) if amax > 0 else np.float32(1.0)
        scales[b] = scale
        y = np.minimum(np.abs(x[rows] / scale), np.float32(E4M3_MAX)) * np.sign(x[rows])   # float32 division
        y = np.where(x[rows] == 0, x[rows], y)                                               # keeps -0.0
        codes[rows] = e4m3_encode(y)
    return codes, scales


def dequantize_blocks(codes, scales, block):
    """float64 [n, D]: code values times the scale of their block."""
    vals = e4m3_decode(codes)
    n = vals.shape[0]
    per_row = np.repeat(np.asarray(scales, dtype=np.float64), block)[:n]
    return vals * per_row[:, None]
