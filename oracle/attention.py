"""Masked softmax attention and its gradient in float64 (test oracle; see oracle/__init__.py).

Eq. 1 of the paper:  Attention(Q, K, V)       = softmax(Q K^T / sqrt(d)) V
Eq. 2 of the paper:  SparseAttention(Q, K, V) = softmax((Q K^T + M) / sqrt(d)) V,
with M in {-inf, 0}^{n x n}; -inf entries are ignored by the softmax.  Because M only
holds -inf and 0, adding it before or after the division by sqrt(d) is the same thing.

All functions work on one (batch, head) slice: Q rows [r, D], K and V [n, D].  Inputs may be
any float dtype (the workloads hand over bf16 values widened to float32); every product,
exponential and sum here is float64.  ``scale`` stands for 1/sqrt(d).

A query row with no visible key has no softmax; the library's ABI defines its output as
O = 0 and LSE = -inf, and the oracle returns the same.
"""
from __future__ import annotations

import numpy as np


def attention_rows(q_rows, k, v, visible, scale):
    """Eq. 2 for the given query rows.

    visible: bool [r, n], True where M = 0.  Returns (O [r, D], LSE [r], P [r, n]).
    """
    q = np.asarray(q_rows, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    m_add = np.where(np.asarray(visible, dtype=bool), 0.0, -np.inf)          # the additive mask M
    logits = (q @ k.T + m_add) * scale
    row_max = logits.max(axis=1, keepdims=True)
    dead = ~np.isfinite(row_max)                                             # rows with no visible key
    row_max = np.where(dead, 0.0, row_max)
    e = np.exp(logits - row_max)                                             # exp(-inf) = 0: ignored
    z = e.sum(axis=1, keepdims=True)
    p = np.divide(e, z, out=np.zeros_like(e), where=z > 0)
    o = p @ v
    with np.errstate(divide="ignore"):
        lse = np.where(dead[:, 0], -np.inf, row_max[:, 0] + np.log(z[:, 0]))
    return o, lse, p


def dense_attention(q, k, v, scale):
    """Eq. 1 (no mask)."""
    vis = np.ones((np.shape(q)[0], np.shape(k)[0]), dtype=bool)
    o, lse, _ = attention_rows(q, k, v, vis, scale)
    return o, lse


def attention_rows_keyset(q_rows, k, v, keys, scale):
    """Eq. 2 for query rows that all see exactly the key set ``keys`` (index array).

    Ignoring the -inf entries means the softmax runs over the visible keys only, so this
    is Eq. 1 on the gathered K[keys], V[keys].  Returns (O [r, D], LSE [r], P [r, len(keys)]).
    """
    keys = np.asarray(keys, dtype=np.int64)
    kk = np.asarray(k)[keys]
    vv = np.asarray(v)[keys]
    vis = np.ones((np.shape(q_rows)[0], keys.size), dtype=bool)
    return attention_rows(q_rows, kk, vv, vis, scale)


def attention_bwd_rows(q_rows, k, v, visible, scale, do_rows):
    """Gradient of L = sum(O * dO) through Eq. 2, for the given query rows.

    With P = softmax rows, O = P V:
        dV = P^T dO,  dP = dO V^T,  D_q = sum_d dO[q,d] O[q,d],
        dS = P * (dP - D),  dQ = scale * dS K,  dK = scale * dS^T Q.
    Returns (dQ [r, D], dK_part [n, D], dV_part [n, D], dS [r, n]); the dK/dV parts are the
    contributions of these query rows only (the full gradient sums them over all rows).
    """
    q = np.asarray(q_rows, dtype=np.float64)
    kk = np.asarray(k, dtype=np.float64)
    vv = np.asarray(v, dtype=np.float64)
    do = np.asarray(do_rows, dtype=np.float64)
    o, _, p = attention_rows(q, kk, vv, visible, scale)
    dv = p.T @ do
    dp = do @ vv.T
    delta = (do * o).sum(axis=1, keepdims=True)
    ds = p * (dp - delta)
    dq = scale * (ds @ kk)
    dk = scale * (ds.T @ q)
    return dq, dk, dv, ds


def attention_bwd_keyset(q_rows, k, v, keys, scale, do_rows, cols=None):
    """Gradient of Eq. 2 for query rows that all see exactly the key set ``keys``.

    Same formulas as attention_bwd_rows on the gathered K[keys], V[keys].  Returns
    (dQ [r, D], dK_part [len(sel), D], dV_part [len(sel), D]) where ``sel`` are the
    positions inside ``keys`` listed in ``cols`` (all of them when cols is None): the dK/dV
    contributions of these query rows to those keys only.  The softmax, O and D_q still run
    over the whole key set."""
    keys = np.asarray(keys, dtype=np.int64)
    q = np.asarray(q_rows, dtype=np.float64)
    kk = np.asarray(k)[keys].astype(np.float64)
    vv = np.asarray(v)[keys].astype(np.float64)
    do = np.asarray(do_rows, dtype=np.float64)
    vis = np.ones((q.shape[0], keys.size), dtype=bool)
    o, _, p = attention_rows(q, kk, vv, vis, scale)
    delta = (do * o).sum(axis=1, keepdims=True)
    dp = do @ vv.T
    ds = p * (dp - delta)
    dq = scale * (ds @ kk)
    sel = np.arange(keys.size) if cols is None else np.asarray(cols, dtype=np.int64)
    dv = p[:, sel].T @ do
    dk = scale * (ds[:, sel].T @ q)
    return dq, dk, dv
