"""Pins of the attention oracle against library routines, identities and finite differences."""
import numpy as np
import pytest
import torch
from scipy.special import logsumexp

from oracle import attention as oa
from oracle import mask as om


def _rand(rng, *shape):
    return rng.standard_normal(shape)


def _mask(rng, r, n, p=0.4):
    vis = rng.random((r, n)) < p
    vis[np.arange(r), rng.integers(0, n, r)] = True      # at least one key per row
    return vis


def test_all_visible_equals_dense_library_attention():
    # Eq. 2 with M = 0 is Eq. 1; Eq. 1 is what torch's scaled_dot_product_attention computes.
    rng = np.random.default_rng(1)
    n, d = 37, 16
    q, k, v = _rand(rng, n, d), _rand(rng, n, d), _rand(rng, n, d)
    scale = 1 / np.sqrt(d)
    o, lse, p = oa.attention_rows(q, k, v, np.ones((n, n), bool), scale)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q)[None], torch.from_numpy(k)[None], torch.from_numpy(v)[None], scale=scale)[0].numpy()
    assert np.allclose(o, ref, rtol=1e-12, atol=1e-13)
    o2, lse2 = oa.dense_attention(q, k, v, scale)
    assert np.array_equal(o, o2) and np.array_equal(lse, lse2)
    assert np.allclose(lse, logsumexp(scale * q @ k.T, axis=1), rtol=1e-13)


def test_masked_equals_library_masked_attention():
    rng = np.random.default_rng(2)
    r, n, d = 23, 41, 8
    q, k, v = _rand(rng, r, d), _rand(rng, n, d), _rand(rng, n, d)
    vis = _mask(rng, r, n)
    o, lse, p = oa.attention_rows(q, k, v, vis, 0.3)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q)[None], torch.from_numpy(k)[None], torch.from_numpy(v)[None],
        attn_mask=torch.from_numpy(vis)[None], scale=0.3)[0].numpy()
    assert np.allclose(o, ref, rtol=1e-12, atol=1e-13)
    logits = np.where(vis, 0.3 * q @ k.T, -np.inf)
    assert np.allclose(lse, logsumexp(logits, axis=1), rtol=1e-13)
    assert (p[~vis] == 0).all()


def test_rows_sum_to_one_and_tv_identity():
    # App. A.2 Eq. (1): ||p~ - p||_1 = 2 Z_out / Z for any mask.
    rng = np.random.default_rng(3)
    f, s, d = 9, 6, 8
    n = f * s
    q, k, v = _rand(rng, n, d), _rand(rng, n, d), _rand(rng, n, d)
    vis = om.flatten_mask(om.token_mask_4d(f, s, 1))
    _, _, p_masked = oa.attention_rows(q, k, v, vis, 0.5)
    _, _, p_dense = oa.attention_rows(q, k, v, np.ones_like(vis), 0.5)
    assert np.allclose(p_masked.sum(1), 1, rtol=1e-13)
    assert np.allclose(p_dense.sum(1), 1, rtol=1e-13)
    a = np.exp(0.5 * q @ k.T)
    z = a.sum(1)
    z_out = (a * ~vis).sum(1)
    assert np.allclose(np.abs(p_masked - p_dense).sum(1), 2 * z_out / z, rtol=1e-10)


def test_special_rows():
    rng = np.random.default_rng(4)
    r, n, d = 5, 11, 4
    q, k, v = _rand(rng, r, d), _rand(rng, n, d), _rand(rng, n, d)
    # exactly one visible key: O is that V row, LSE is that logit
    vis = np.zeros((r, n), bool)
    pick = np.array([0, 3, 10, 7, 7])
    vis[np.arange(r), pick] = True
    o, lse, _ = oa.attention_rows(q, k, v, vis, 0.7)
    assert np.allclose(o, v[pick], rtol=1e-14)
    assert np.allclose(lse, 0.7 * (q * k[pick]).sum(1), rtol=1e-13)
    # no visible key: O = 0, LSE = -inf
    vis[2] = False
    o, lse, p = oa.attention_rows(q, k, v, vis, 0.7)
    assert (o[2] == 0).all() and lse[2] == -np.inf and (p[2] == 0).all()
    # constant V => constant O; a key-independent shift of the logits leaves O unchanged
    vis = _mask(rng, r, n)
    o, _, _ = oa.attention_rows(q, k, np.full((n, d), 2.5), vis, 0.7)
    assert np.allclose(o, 2.5, rtol=1e-14)
    k1 = np.concatenate([k, np.ones((n, 1))], axis=1)
    qa = np.concatenate([q, np.zeros((r, 1))], axis=1)
    qb = np.concatenate([q, np.full((r, 1), 3.0)], axis=1)     # adds 3 to every logit of the row
    oa_, la, _ = oa.attention_rows(qa, k1, v, vis, 0.7)
    ob_, lb, _ = oa.attention_rows(qb, k1, v, vis, 0.7)
    assert np.allclose(oa_, ob_, rtol=1e-12) and np.allclose(lb - la, 0.7 * 3.0, rtol=1e-12)


def test_keyset_form_equals_bool_form():
    rng = np.random.default_rng(5)
    r, n, d = 6, 50, 8
    q, k, v = _rand(rng, r, d), _rand(rng, n, d), _rand(rng, n, d)
    keys = np.array([1, 2, 3, 17, 18, 40, 49])
    vis = np.zeros((r, n), bool)
    vis[:, keys] = True
    o1, l1, p1 = oa.attention_rows(q, k, v, vis, 0.35)
    o2, l2, p2 = oa.attention_rows_keyset(q, k, v, keys, 0.35)
    assert np.allclose(o1, o2, rtol=1e-13) and np.allclose(l1, l2, rtol=1e-13)
    assert np.allclose(p1[:, keys], p2, rtol=1e-13)


def test_large_logits_do_not_overflow():
    q = np.array([[300.0, 0.0]])
    k = np.array([[3.0, 0.0], [2.0, 0.0], [-5.0, 1.0]])
    v = np.eye(3)[:, :2]
    o, lse, p = oa.attention_rows(q, k, v, np.ones((1, 3), bool), 1.0)
    assert np.isfinite(o).all() and np.isclose(lse[0], 900 + np.log1p(np.exp(-300.0)))


# ---- gradient ---------------------------------------------------------------------------------

def _loss(q, k, v, vis, scale, g):
    o, _, _ = oa.attention_rows(q, k, v, vis, scale)
    return float((o * g).sum())


def test_backward_finite_differences():
    rng = np.random.default_rng(6)
    f, s, d = 5, 3, 4
    n = f * s
    q, k, v, g = _rand(rng, n, d), _rand(rng, n, d), _rand(rng, n, d), _rand(rng, n, d)
    vis = om.flatten_mask(om.token_mask_4d(f, s, 1))
    scale = 0.5
    dq, dk, dv, ds = oa.attention_bwd_rows(q, k, v, vis, scale, g)
    assert np.allclose(ds.sum(1), 0, atol=1e-13)              # softmax Jacobian rows sum to zero
    assert (ds[~vis] == 0).all()
    eps = 1e-6
    for name, arr, grad in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        num = np.zeros_like(arr)
        for idx in np.ndindex(*arr.shape):
            old = arr[idx]
            arr[idx] = old + eps
            lp = _loss(q, k, v, vis, scale, g)
            arr[idx] = old - eps
            lm = _loss(q, k, v, vis, scale, g)
            arr[idx] = old
            num[idx] = (lp - lm) / (2 * eps)
        assert np.allclose(grad, num, rtol=1e-6, atol=1e-8), name


def test_backward_equals_library_autograd():
    rng = np.random.default_rng(7)
    r, n, d = 13, 29, 8
    q, k, v, g = _rand(rng, r, d), _rand(rng, n, d), _rand(rng, n, d), _rand(rng, r, d)
    vis = _mask(rng, r, n)
    dq, dk, dv, _ = oa.attention_bwd_rows(q, k, v, vis, 0.25, g)
    tq, tk, tv = (torch.from_numpy(x).clone().requires_grad_(True) for x in (q, k, v))
    out = torch.nn.functional.scaled_dot_product_attention(
        tq[None], tk[None], tv[None], attn_mask=torch.from_numpy(vis)[None], scale=0.25)[0]
    (out * torch.from_numpy(g)).sum().backward()
    assert np.allclose(dq, tq.grad.numpy(), rtol=1e-11, atol=1e-13)
    assert np.allclose(dk, tk.grad.numpy(), rtol=1e-11, atol=1e-13)
    assert np.allclose(dv, tv.grad.numpy(), rtol=1e-11, atol=1e-13)


def test_backward_row_parts_add_up():
    rng = np.random.default_rng(8)
    r, n, d = 10, 17, 4
    q, k, v, g = _rand(rng, r, d), _rand(rng, n, d), _rand(rng, n, d), _rand(rng, r, d)
    vis = _mask(rng, r, n)
    dq, dk, dv, _ = oa.attention_bwd_rows(q, k, v, vis, 0.4, g)
    dq1, dk1, dv1, _ = oa.attention_bwd_rows(q[:4], k, v, vis[:4], 0.4, g[:4])
    dq2, dk2, dv2, _ = oa.attention_bwd_rows(q[4:], k, v, vis[4:], 0.4, g[4:])
    assert np.allclose(np.concatenate([dq1, dq2]), dq, rtol=1e-13)
    assert np.allclose(dk1 + dk2, dk, rtol=1e-12, atol=1e-14) and np.allclose(dv1 + dv2, dv, rtol=1e-12, atol=1e-14)


def test_backward_keyset_form_equals_bool_form():
    rng = np.random.default_rng(9)
    r, n, d = 7, 40, 8
    q, k, v, g = _rand(rng, r, d), _rand(rng, n, d), _rand(rng, n, d), _rand(rng, r, d)
    keys = np.array([0, 1, 5, 6, 7, 20, 21, 39])
    vis = np.zeros((r, n), bool)
    vis[:, keys] = True
    dq, dk, dv, _ = oa.attention_bwd_rows(q, k, v, vis, 0.3, g)
    dq2, dk2, dv2 = oa.attention_bwd_keyset(q, k, v, keys, 0.3, g)
    assert np.allclose(dq, dq2, rtol=1e-12, atol=1e-14)
    assert np.allclose(dk[keys], dk2, rtol=1e-12, atol=1e-14) and np.allclose(dv[keys], dv2, rtol=1e-12, atol=1e-14)
    assert (dk[np.setdiff1d(np.arange(n), keys)] == 0).all()
    dq3, dk3, dv3 = oa.attention_bwd_keyset(q, k, v, keys, 0.3, g, cols=[2, 3, 4])
    assert np.allclose(dq3, dq2) and np.allclose(dk3, dk2[2:5]) and np.allclose(dv3, dv2[2:5])
