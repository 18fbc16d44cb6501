"""Text tokens appended to the video sequence (they see and are seen by every token): lists
bit-exact against the brute-force oracle, attention against Eq. 2 under the extended mask
(run with -m gpu)."""
import numpy as np
import pytest
import torch

from oracle import attention as oa
from oracle import build as obuild
from oracle import mask as om
from paper_2506_19852_amd import binding as rb

from util import assert_close

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("f,s,block,sink,extra", [
    (33, 40, 64, 1, 77), (16, 100, 128, 1, 256), (5, 1000, 128, 0, 1), (64, 24, 128, 2, 300), (3, 129, 64, 1, 64),
    (1, 1, 64, 1, 5),
])
def test_lists_bit_exact(f, s, block, sink, extra):
    print(f"text tokens mask f={f} s={s} block={block} sink={sink} extra={extra}", flush=True)
    bitmap, _ = obuild.mask_scan(f, s, block, sink, 0, None, 1, 1, extra)
    want_ptr, want_idx = om.block_lists(bitmap)
    m = rb.radial_mask_build(f, s, block, sink, rb.RADIAL_MASK_TRANSPOSE, extra_tokens=extra)
    assert rb.radial_mask_info(m)["n_tokens"] == f * s + extra
    got_ptr, got_idx = rb.radial_mask_copy_to_host(m)
    assert np.array_equal(got_ptr, want_ptr) and np.array_equal(got_idx, want_idx)
    t_ptr, t_idx = rb.radial_mask_copy_transpose_to_host(m)
    wt_ptr, wt_idx = om.block_lists(np.ascontiguousarray(bitmap.T))
    assert np.array_equal(t_ptr, wt_ptr) and np.array_equal(t_idx, wt_idx)
    m.free()


def test_negative_extra_is_rejected():
    with pytest.raises(rb.RadialError) as e:
        rb.radial_mask_build(4, 64, 64, 1, 0, extra_tokens=-1)
    assert e.value.code == -1


def _randn_bf16(shape, seed):
    g = torch.Generator(device="cpu").manual_seed(seed)
    return torch.randn(shape, generator=g).to(torch.bfloat16).to(DEV)


@pytest.mark.parametrize("exact", [False, True])
@pytest.mark.parametrize("f,s,block,D,extra", [(12, 150, 128, 128, 200), (20, 64, 64, 64, 30), (9, 200, 128, 64, 256)])
def test_attention_with_text_tokens(f, s, block, D, extra, exact):
    print(f"text tokens attention f={f} s={s} block={block} D={D} extra={extra} token rule={exact}", flush=True)
    N = f * s + extra
    q, k, v, do = (_randn_bf16((1, 1, N, D), 95 + i) for i in range(4))
    scale = 1.0 / np.sqrt(D)
    flags = rb.RADIAL_MASK_TRANSPOSE | (rb.RADIAL_MASK_TOKEN_EXACT if exact else 0)
    mask = rb.radial_mask_build(f, s, block, 1, flags, extra_tokens=extra)
    out = torch.empty_like(q)
    lse = torch.empty((1, 1, N), dtype=torch.float32, device=DEV)
    rb.radial_attn_fwd(q, k, v, out, lse, mask, scale)
    ws = torch.empty(rb.radial_attn_bwd_workspace(1, 1, N, D, mask), dtype=torch.uint8, device=DEV)
    dq, dk, dv = (torch.full_like(q, float("nan")) for _ in range(3))
    rb.radial_attn_bwd(q, k, v, out, do, lse, dq, dk, dv, mask, scale, ws)
    torch.cuda.synchronize()
    if exact:
        vis = om.token_mask_rows_with_text(f, s, 1, np.arange(N), extra)
    else:
        bitmap, _ = obuild.mask_scan(f, s, block, 1, 0, None, 1, 1, extra)
        vis = np.repeat(np.repeat(bitmap, block, axis=0), block, axis=1)[:N, :N]
    qh, kh, vh, gh = (t[0, 0].float().cpu().numpy() for t in (q, k, v, do))
    ref_o, ref_l, _ = oa.attention_rows(qh, kh, vh, vis, scale)
    assert_close(out[0, 0].float().cpu().numpy(), ref_o, "O")
    assert np.allclose(lse[0, 0].cpu().numpy(), ref_l, rtol=1e-4, atol=1e-4)
    ref = oa.attention_bwd_rows(qh, kh, vh, vis, scale, gh)[:3]
    for got, want, nm in zip((dq, dk, dv), ref, ("dQ", "dK", "dV")):
        assert_close(got[0, 0].float().cpu().numpy(), want, nm)
    mask.free()
