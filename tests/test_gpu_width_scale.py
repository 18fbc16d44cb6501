"""Sparsity knob (width scale c = width_num/width_den on frame distances >= 2): GPU mask builder
bit-exact against the brute-force oracle, and the token rule under the knob (run with -m gpu)."""
import numpy as np
import pytest
import torch

from oracle import attention as oa
from oracle import build as obuild
from oracle import mask as om
from paper_2506_19852_amd import binding as rb
from paper_2506_19852_amd import workloads as wl

from util import assert_close, sample_qblocks

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

SCALES = [(1, 2), (2, 3), (13, 20), (3, 2), (1, 7), (5, 1), (1, 300)]


@pytest.mark.parametrize("num,den", SCALES)
@pytest.mark.parametrize("f,s,block,sink", [
    (300, 2, 64, 1), (100, 7, 64, 0), (33, 40, 128, 1), (16, 100, 64, 1), (5, 1000, 128, 2), (64, 24, 128, 0),
    (700, 3, 128, 1), (40, 130, 64, 1), (3, 129, 128, 1),
])
def test_mask_bit_exact(f, s, block, sink, num, den):
    print(f"width scale mask f={f} s={s} block={block} sink={sink} c={num}/{den}", flush=True)
    bitmap, _ = obuild.mask_scan(f, s, block, sink, 0, None, num, den)
    want_ptr, want_idx = om.block_lists(bitmap)
    m = rb.radial_mask_build(f, s, block, sink, rb.RADIAL_MASK_TRANSPOSE, width_num=num, width_den=den)
    got_ptr, got_idx = rb.radial_mask_copy_to_host(m)
    assert np.array_equal(got_ptr, want_ptr) and np.array_equal(got_idx, want_idx)
    t_ptr, t_idx = rb.radial_mask_copy_transpose_to_host(m)
    wt_ptr, wt_idx = om.block_lists(np.ascontiguousarray(bitmap.T))
    assert np.array_equal(t_ptr, wt_ptr) and np.array_equal(t_idx, wt_idx)
    m.free()


def test_parameter_errors():
    for num, den in ((0, 1), (1, 0), (40000, 1), (1, 40000), (-1, 1)):
        with pytest.raises(rb.RadialError) as e:
            rb.radial_mask_build(4, 64, 64, 1, 0, width_num=num, width_den=den)
        assert e.value.code == -1
    with pytest.raises(rb.RadialError) as e:                    # tokens_per_frame * width_num >= 2^31
        rb.radial_mask_build(1, 100000, 64, 1, 0, width_num=30000, width_den=1)
    assert e.value.code == -1


@pytest.mark.parametrize("name,num,den,nsample", [
    ("cfg3_hunyuan720p", 13, 20, 24),
    ("cfg4_hunyuan720p_4x", 13, 20, 10),
    ("cfg2_wan480p", 1, 2, 40),
])
def test_workload_masks_sampled_rows(name, num, den, nsample):
    """Full-size lists under the knob: sampled query blocks against the brute-force scan."""
    w = wl.WORKLOADS[name]
    f, s, block = w.frames, w.tokens_per_frame, w.block
    print(f"width scale workload mask {name} c={num}/{den}", flush=True)
    m = rb.radial_mask_build(f, s, block, 1, 0, width_num=num, width_den=den)
    ptr, idx = rb.radial_mask_copy_to_host(m)
    base = rb.radial_mask_build(f, s, block, 1)
    bptr, _ = rb.radial_mask_copy_to_host(base)
    assert ptr[-1] < bptr[-1]                                   # c < 1 lists fewer pairs
    nb = ptr.size - 1
    for qb in sample_qblocks(nb, np.diff(ptr), s, block, nsample, w.seed + 3):
        bm, _ = obuild.mask_scan(f, s, block, 1, qb, qb + 1, num, den)
        assert np.array_equal(idx[ptr[qb]:ptr[qb + 1]], np.flatnonzero(bm[0])), qb
    m.free()
    base.free()


def _randn_bf16(shape, seed, scale=1.0):
    g = torch.Generator(device="cpu").manual_seed(seed)
    return (torch.randn(shape, generator=g) * scale).to(torch.bfloat16).to(DEV)


@pytest.mark.parametrize("f,s,block,D,sink,num,den", [
    (9, 150, 128, 128, 1, 13, 20),
    (33, 64, 64, 64, 1, 1, 2),
    (20, 100, 128, 64, 0, 3, 2),        # c > 1: wider diagonals, clipped at the frame
    (40, 70, 64, 128, 1, 1, 40),        # widths below one: sub-sampled single diagonals
])
def test_token_rule_forward_backward(f, s, block, D, sink, num, den):
    print(f"width scale token rule f={f} s={s} block={block} D={D} c={num}/{den}", flush=True)
    N = f * s
    q, k, v, do = (_randn_bf16((1, 1, N, D), 51 + i) for i in range(4))
    scale = 1.0 / np.sqrt(D)
    mask = rb.radial_mask_build(f, s, block, sink, rb.RADIAL_MASK_TRANSPOSE | rb.RADIAL_MASK_TOKEN_EXACT,
                                width_num=num, width_den=den)
    out = torch.empty_like(q)
    lse = torch.empty((1, 1, N), dtype=torch.float32, device=DEV)
    rb.radial_attn_fwd(q, k, v, out, lse, mask, scale)
    ws = torch.empty(rb.radial_attn_bwd_workspace(1, 1, N, D, mask), dtype=torch.uint8, device=DEV)
    dq, dk, dv = (torch.full_like(q, float("nan")) for _ in range(3))
    rb.radial_attn_bwd(q, k, v, out, do, lse, dq, dk, dv, mask, scale, ws)
    torch.cuda.synchronize()
    qh, kh, vh, gh = (t[0, 0].float().cpu().numpy() for t in (q, k, v, do))
    vis = om.token_mask_rows(f, s, sink, np.arange(N), num, den)
    ref_o, ref_l, _ = oa.attention_rows(qh, kh, vh, vis, scale)
    assert_close(out[0, 0].float().cpu().numpy(), ref_o, "O")
    assert np.allclose(lse[0, 0].cpu().numpy(), ref_l, rtol=1e-4, atol=1e-4)
    ref = oa.attention_bwd_rows(qh, kh, vh, vis, scale, gh)[:3]
    for got, want, nm in zip((dq, dk, dv), ref, ("dQ", "dK", "dV")):
        assert_close(got[0, 0].float().cpu().numpy(), want, nm)
    mask.free()


def test_block_dense_forward_under_the_knob():
    f, s, block, D, num, den = 12, 200, 128, 128, 13, 20
    print("width scale block-dense forward", flush=True)
    N = f * s
    q, k, v = (_randn_bf16((1, 2, N, D), 61 + i) for i in range(3))
    scale = 1.0 / np.sqrt(D)
    mask = rb.radial_mask_build(f, s, block, 1, 0, width_num=num, width_den=den)
    out = torch.empty_like(q)
    lse = torch.empty((1, 2, N), dtype=torch.float32, device=DEV)
    rb.radial_attn_fwd(q, k, v, out, lse, mask, scale)
    torch.cuda.synchronize()
    bitmap, _ = obuild.mask_scan(f, s, block, 1, 0, None, num, den)
    vis = np.repeat(np.repeat(bitmap, block, axis=0), block, axis=1)[:N, :N]
    for h in range(2):
        qh, kh, vh = (t[0, h].float().cpu().numpy() for t in (q, k, v))
        ref_o, ref_l, _ = oa.attention_rows(qh, kh, vh, vis, scale)
        assert_close(out[0, h].float().cpu().numpy(), ref_o, f"h{h} O")
        assert np.allclose(lse[0, h].cpu().numpy(), ref_l, rtol=1e-4, atol=1e-4)
    mask.free()
