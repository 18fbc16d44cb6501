"""Token-exact masking inside listed blocks: the GPU path under RADIAL_MASK_TOKEN_EXACT vs
Eq. 2 evaluated by the float64 oracle with the token mask of Sec. 4.2 itself (run with -m gpu)."""
import numpy as np
import pytest
import torch

from oracle import attention as oa
from oracle import build as obuild
from oracle import mask as om
from paper_2506_19852_amd import binding as rb
from paper_2506_19852_amd import workloads as wl

from util import assert_close, backward_rounding_bounds, sample_qblocks

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
EXACT = rb.RADIAL_MASK_TOKEN_EXACT


def _randn_bf16(shape, seed, scale=1.0):
    g = torch.Generator(device="cpu").manual_seed(seed)
    return (torch.randn(shape, generator=g) * scale).to(torch.bfloat16).to(DEV)


def _check_fwd_blocks(out, lse, q, k, v, f, s, sink, block, qblocks, scale, pairs, what):
    n = f * s
    worst = 0.0
    for (b, h) in pairs:
        qh, kh, vh = (t[b, h].float().cpu().numpy() for t in (q, k, v))
        oh = out[b, h].float().cpu().numpy()
        lh = lse[b, h].cpu().numpy()
        for qb in qblocks:
            rows = np.arange(qb * block, min(n, (qb + 1) * block))
            vis = obuild.token_mask(f, s, sink, int(rows[0]), int(rows[-1]) + 1, np.arange(n))
            ref_o, ref_l, _ = oa.attention_rows(qh[rows], kh, vh, vis, scale)
            err, _ = assert_close(oh[rows], ref_o, f"{what} b{b} h{h} qb{qb} O")
            worst = max(worst, err)
            assert np.isfinite(ref_l).all()                     # every token sees itself
            assert np.allclose(lh[rows], ref_l, rtol=1e-4, atol=1e-4), f"{what} b{b} h{h} qb{qb} LSE"
    return worst


@pytest.mark.parametrize("f,s,block,D,B,H,sink,qscale", [
    (5, 200, 128, 128, 1, 2, 1, 1.0),      # blocks straddle frames, ragged last block
    (5, 200, 64, 64, 2, 1, 0, 1.0),
    (3, 333, 128, 64, 1, 2, 1, 1.0),
    (7, 100, 64, 128, 1, 1, 2, 1.0),
    (9, 150, 128, 128, 1, 2, 1, 6.0),      # peaked rows
    (33, 64, 128, 128, 1, 1, 1, 1.0),      # two frames per block, widths down to 2
    (150, 64, 64, 64, 1, 1, 1, 1.0),       # frame distances >= 2s: sub-sampled single diagonals
    (40, 70, 128, 64, 1, 1, 0, 1.0),       # frame length coprime to the block
    (1, 65, 64, 64, 1, 1, 1, 1.0),
])
def test_forward_small(f, s, block, D, B, H, sink, qscale):
    print(f"token-exact fwd f={f} s={s} block={block} D={D} sink={sink}", flush=True)
    N = f * s
    q = _randn_bf16((B, H, N, D), 31, qscale)
    k = _randn_bf16((B, H, N, D), 32)
    v = _randn_bf16((B, H, N, D), 33)
    scale = 1.0 / np.sqrt(D)
    mask = rb.radial_mask_build(f, s, block, sink, EXACT)
    # the block lists do not depend on the flag
    plain = rb.radial_mask_build(f, s, block, sink)
    for a, b in zip(rb.radial_mask_copy_to_host(mask), rb.radial_mask_copy_to_host(plain)):
        assert np.array_equal(a, b)
    out = torch.full_like(q, float("nan"))
    lse = torch.full(q.shape[:3], float("nan"), dtype=torch.float32, device=DEV)
    rb.radial_attn_fwd(q, k, v, out, lse, mask, scale)
    torch.cuda.synchronize()
    nb = -(-N // block)
    pairs = [(b, h) for b in range(B) for h in range(H)]
    _check_fwd_blocks(out, lse, q, k, v, f, s, sink, block, range(nb), scale, pairs, "exact small")
    # and it differs from the block-dense result wherever a listed block is partly masked
    if f > 2:
        out_d = torch.empty_like(q)
        rb.radial_attn_fwd(q, k, v, out_d, None, plain, scale)
        torch.cuda.synchronize()
        assert not torch.equal(out, out_d)
    mask.free()
    plain.free()


def test_flag_errors():
    with pytest.raises(rb.RadialError) as e:
        rb.radial_mask_build(4, 32, 64, 1, EXACT)               # frames shorter than a stage of keys
    assert e.value.code == -4
    with pytest.raises(rb.RadialError) as e:
        rb.radial_mask_build_dense(256, 64, EXACT)
    assert e.value.code == -1
    rp = np.array([0, 1], dtype=np.int32)
    ci = np.array([0], dtype=np.int32)
    with pytest.raises(rb.RadialError) as e:
        rb.radial_mask_from_csr(64, 64, rp, ci, EXACT)
    assert e.value.code == -1


@pytest.mark.parametrize("name,heads,nsample", [
    ("cfg2_wan480p", (3,), 48),
    ("cfg3_hunyuan720p", (11,), 32),
])
def test_workload_forward(name, heads, nsample):
    w = wl.WORKLOADS[name]
    print(f"token-exact fwd workload {name}", flush=True)
    f, s, block = w.frames, w.tokens_per_frame, w.block
    x = {nm: wl.make_tensor(w, nm, DEV) for nm in ("q", "k", "v")}
    mask = rb.radial_mask_build(f, s, block, 1, EXACT)
    row_ptr, _ = rb.radial_mask_copy_to_host(mask)
    nb = row_ptr.size - 1
    out = torch.full_like(x["q"], float("nan"))
    lse = torch.full(x["q"].shape[:3], float("nan"), dtype=torch.float32, device=DEV)
    rb.radial_attn_fwd(x["q"], x["k"], x["v"], out, lse, mask, w.scale)
    torch.cuda.synchronize()
    qblocks = sample_qblocks(nb, np.diff(row_ptr), s, block, nsample, w.seed + 1)
    worst = _check_fwd_blocks(out, lse, x["q"], x["k"], x["v"], f, s, 1, block, qblocks, w.scale,
                              [(0, h) for h in heads], name)
    print(f"{name}: {len(qblocks)} query blocks checked, max |err| {worst:.3e}", flush=True)
    assert torch.isfinite(out.float()).all() and torch.isfinite(lse).all()
    mask.free()


# ---- backward ---------------------------------------------------------------------------------

def _fwd_bwd(q, k, v, do, mask, scale):
    B, H, N, D = q.shape
    out = torch.empty_like(q)
    lse = torch.empty((B, H, N), dtype=torch.float32, device=q.device)
    rb.radial_attn_fwd(q, k, v, out, lse, mask, scale)
    ws = torch.empty(rb.radial_attn_bwd_workspace(B, H, N, D, mask), dtype=torch.uint8, device=q.device)
    ws.fill_(0xFF)
    dq, dk, dv = (torch.full_like(q, float("nan")) for _ in range(3))
    rb.radial_attn_bwd(q, k, v, out, do, lse, dq, dk, dv, mask, scale, ws)
    torch.cuda.synchronize()
    return out, lse, dq, dk, dv


@pytest.mark.parametrize("f,s,block,D,B,H,sink,qscale", [
    (5, 200, 128, 128, 1, 2, 1, 1.0),
    (5, 200, 64, 64, 2, 1, 0, 1.0),
    (3, 333, 128, 64, 1, 1, 1, 1.0),
    (7, 100, 64, 128, 1, 1, 2, 1.0),
    (9, 150, 128, 128, 1, 1, 1, 4.0),      # peaked rows
    (33, 64, 128, 128, 1, 1, 1, 1.0),
    (130, 64, 64, 64, 1, 1, 1, 1.0),       # includes the sub-sampled single diagonals
    (40, 70, 128, 64, 1, 1, 0, 1.0),
    (1, 65, 64, 64, 1, 1, 1, 1.0),
])
def test_backward_small(f, s, block, D, B, H, sink, qscale):
    print(f"token-exact bwd f={f} s={s} block={block} D={D} sink={sink}", flush=True)
    N = f * s
    q = _randn_bf16((B, H, N, D), 41, qscale)
    k, v, do = (_randn_bf16((B, H, N, D), 42 + i) for i in range(3))
    scale = 1.0 / np.sqrt(D)
    mask = rb.radial_mask_build(f, s, block, sink, rb.RADIAL_MASK_TRANSPOSE | EXACT)
    _, _, dq, dk, dv = _fwd_bwd(q, k, v, do, mask, scale)
    vis = obuild.token_mask(f, s, sink, 0, N, np.arange(N))
    for b in range(B):
        for h in range(H):
            qh, kh, vh, gh = (t[b, h].float().cpu().numpy() for t in (q, k, v, do))
            ref, bounds = backward_rounding_bounds(qh, kh, vh, vis, scale, gh)
            for got, want, bound, nm in zip((dq, dk, dv), ref, bounds, ("dQ", "dK", "dV")):
                assert_close(got[b, h].float().cpu().numpy(), want, f"exact b{b} h{h} {nm}",
                             extra_atol=2.0 * bound if qscale != 1.0 else None)
    mask.free()


def test_workload_backward(capsys):
    """Forward+backward workload at full size under the token rule: dQ of sampled query blocks
    and dK/dV of one key block, each against the oracle with the token mask."""
    w = wl.WORKLOADS["cfg5_wan480p_4x_bwd"]
    print("token-exact bwd workload cfg5", flush=True)
    f, s, block = w.frames, w.tokens_per_frame, w.block
    x = wl.make_inputs(w, DEV)
    mask = rb.radial_mask_build(f, s, block, 1, rb.RADIAL_MASK_TRANSPOSE | EXACT)
    out, lse, dq, dk, dv = _fwd_bwd(x["q"], x["k"], x["v"], x["do"], mask, w.scale)
    head = 9
    qh, kh, vh, gh = (x[n][0, head].float().cpu().numpy() for n in ("q", "k", "v", "do"))
    nb = -(-w.N // block)

    def block_grads(qb):
        """dQ of query block qb and its dK/dV contributions, on the keys it can see."""
        rows = np.arange(qb * block, min(w.N, (qb + 1) * block))
        listed, _ = obuild.mask_scan(f, s, block, 1, qb, qb + 1)          # candidate key blocks
        cand = np.flatnonzero(om.expand_block_row(listed[0], block, w.N))
        vis = obuild.token_mask(f, s, 1, int(rows[0]), int(rows[-1]) + 1, cand)
        keep = vis.any(axis=0)
        keys, vis = cand[keep], vis[:, keep]
        g_q, g_k, g_v, _ = oa.attention_bwd_rows(qh[rows], kh[keys], vh[keys], vis, w.scale, gh[rows])
        return rows, keys, g_q, g_k, g_v

    rng = np.random.default_rng(w.seed + 2)
    for qb in sorted({0, nb - 1, s // block, *rng.integers(0, nb, 5).tolist()}):
        rows, _, ref_dq, _, _ = block_grads(qb)
        assert_close(dq[0, head, rows[0]:rows[-1] + 1].float().cpu().numpy(), ref_dq, f"exact cfg5 dQ qb{qb}")
    # which query blocks list key block kb comes from the oracle's own block mask (a query block the
    # library's transposed list had dropped would otherwise be missing from both sides)
    bitmap, _ = obuild.mask_scan(f, s, block, 1)
    col_len = bitmap.sum(axis=0)
    kb = int(np.argmin(col_len[nb // 4: 3 * nb // 4])) + nb // 4              # the shortest column of the middle half
    kcols = np.arange(kb * block, min(w.N, (kb + 1) * block))
    ref_dk = np.zeros((kcols.size, w.D))
    ref_dv = np.zeros((kcols.size, w.D))
    listers = np.flatnonzero(bitmap[:, kb])
    assert listers.size > 128                                               # the kernel reloads its list chunk
    for n_done, qb in enumerate(listers):
        _, keys, _, g_k, g_v = block_grads(int(qb))
        pos = np.searchsorted(keys, kcols)
        hit = (pos < keys.size) & (keys[np.minimum(pos, keys.size - 1)] == kcols)
        ref_dk[hit] += g_k[pos[hit]]
        ref_dv[hit] += g_v[pos[hit]]
        if n_done % 50 == 49:
            with capsys.disabled():                                     # a sign of life for whoever watches the run
                print(f" [cfg5 token-rule dK/dV: {n_done + 1}/{len(listers)} query blocks summed]", flush=True)
    assert_close(dk[0, head, kcols[0]:kcols[-1] + 1].float().cpu().numpy(), ref_dk, f"exact cfg5 dK kb{kb}")
    assert_close(dv[0, head, kcols[0]:kcols[-1] + 1].float().cpu().numpy(), ref_dv, f"exact cfg5 dV kb{kb}")
    print(f"cfg5 key block {kb}: {len(listers)} query blocks summed by the oracle", flush=True)
    for t in (dq, dk, dv):
        assert torch.isfinite(t.float()).all()
    mask.free()
