"""Other static masks through the library: the banded builder bit-exact against the oracle's
definition, attention under those lists and under their token rule, and a pattern that only the
caller-supplied-list interface can express (run with -m gpu)."""
import numpy as np
import pytest
import torch

from oracle import attention as oa
from oracle import mask as om
from oracle import patterns as op
from paper_2506_19852_amd import binding as rb

from util import assert_close

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _tables(f, s):
    return {
        "spatial": op.half_widths_spatial(f, s, 1),
        "temporal": op.half_widths_temporal(f, s, 40),
        "sliding": op.half_widths_sliding(f, s, 2, 60),
        "harmonic": op.half_widths_harmonic(f, s),
    }


@pytest.mark.parametrize("pattern", ["spatial", "temporal", "sliding", "harmonic"])
@pytest.mark.parametrize("f,s,block,sink", [(12, 200, 128, 1), (30, 70, 64, 0), (5, 333, 128, 1), (64, 24, 64, 2)])
def test_banded_lists_bit_exact(pattern, f, s, block, sink):
    print(f"banded {pattern} f={f} s={s} block={block} sink={sink}", flush=True)
    hw = _tables(f, s)[pattern]
    n = f * s
    bitmap = op.block_bitmap(lambda rows: op.banded_mask_rows(f, s, sink, hw, rows), n, block)
    want_ptr, want_idx = om.block_lists(bitmap)
    m = rb.radial_mask_build_banded(f, s, block, sink, hw, rb.RADIAL_MASK_TRANSPOSE)
    got_ptr, got_idx = rb.radial_mask_copy_to_host(m)
    assert np.array_equal(got_ptr, want_ptr) and np.array_equal(got_idx, want_idx)
    t_ptr, t_idx = rb.radial_mask_copy_transpose_to_host(m)
    wt_ptr, wt_idx = om.block_lists(np.ascontiguousarray(bitmap.T))
    assert np.array_equal(t_ptr, wt_ptr) and np.array_equal(t_idx, wt_idx)
    m.free()


@pytest.mark.parametrize("f,s,block,sink", [(12, 200, 128, 1), (20, 64, 64, 0), (3, 129, 128, 1)])
def test_banded_radial_table_reproduces_the_radial_builder(f, s, block, sink):
    hw = op.half_widths_radial(f, s)
    a = rb.radial_mask_build_banded(f, s, block, sink, hw)
    b = rb.radial_mask_build(f, s, block, sink)
    for x, y in zip(rb.radial_mask_copy_to_host(a), rb.radial_mask_copy_to_host(b)):
        assert np.array_equal(x, y)
    a.free()
    b.free()


def test_argument_errors():
    with pytest.raises(ValueError):
        rb.radial_mask_build_banded(4, 64, 64, 1, [1, 2, 3])
    with pytest.raises(rb.RadialError) as e:
        rb.radial_mask_build_banded(4, 32, 64, 1, [1, 2, 3, 4], rb.RADIAL_MASK_TOKEN_EXACT)
    assert e.value.code == -4
    with pytest.raises(rb.RadialError) as e:
        rb.radial_mask_build_banded(4, 64, 100, 1, [1, 2, 3, 4])
    assert e.value.code == -4


def _randn_bf16(shape, seed):
    g = torch.Generator(device="cpu").manual_seed(seed)
    return torch.randn(shape, generator=g).to(torch.bfloat16).to(DEV)


def _attention_all(q, k, v, do, mask, scale):
    B, H, N, D = q.shape
    out = torch.empty_like(q)
    lse = torch.empty((B, H, N), dtype=torch.float32, device=DEV)
    rb.radial_attn_fwd(q, k, v, out, lse, mask, scale)
    ws = torch.empty(rb.radial_attn_bwd_workspace(B, H, N, D, mask), dtype=torch.uint8, device=DEV)
    dq, dk, dv = (torch.full_like(q, float("nan")) for _ in range(3))
    rb.radial_attn_bwd(q, k, v, out, do, lse, dq, dk, dv, mask, scale, ws)
    torch.cuda.synchronize()
    return out, lse, dq, dk, dv


def _check_against(vis, q, k, v, do, scale, got):
    out, lse, dq, dk, dv = got
    qh, kh, vh, gh = (t[0, 0].float().cpu().numpy() for t in (q, k, v, do))
    ref_o, ref_l, _ = oa.attention_rows(qh, kh, vh, vis, scale)
    assert_close(out[0, 0].float().cpu().numpy(), ref_o, "O")
    fin = np.isfinite(ref_l)
    assert np.allclose(lse[0, 0].cpu().numpy()[fin], ref_l[fin], rtol=1e-4, atol=1e-4)
    ref = oa.attention_bwd_rows(qh, kh, vh, vis, scale, gh)[:3]
    for g, want, nm in zip((dq, dk, dv), ref, ("dQ", "dK", "dV")):
        assert_close(g[0, 0].float().cpu().numpy(), want, nm)


@pytest.mark.parametrize("pattern", ["spatial", "temporal", "sliding", "harmonic"])
@pytest.mark.parametrize("exact", [False, True])
def test_attention_under_banded_masks(pattern, exact):
    f, s, block, D, sink = 14, 150, 128, 128, 1
    print(f"banded attention {pattern} token rule={exact}", flush=True)
    N = f * s
    hw = _tables(f, s)[pattern]
    q, k, v, do = (_randn_bf16((1, 1, N, D), 71 + i) for i in range(4))
    scale = 1.0 / np.sqrt(D)
    flags = rb.RADIAL_MASK_TRANSPOSE | (rb.RADIAL_MASK_TOKEN_EXACT if exact else 0)
    mask = rb.radial_mask_build_banded(f, s, block, sink, hw, flags)
    got = _attention_all(q, k, v, do, mask, scale)
    token = op.banded_mask_rows(f, s, sink, hw, np.arange(N))
    if exact:
        vis = token
    else:                                                  # block-dense inside the listed blocks
        bitmap = op.block_bitmap(lambda rows: token[rows], N, block)
        vis = np.repeat(np.repeat(bitmap, block, axis=0), block, axis=1)[:N, :N]
    _check_against(vis, q, k, v, do, scale, got)
    mask.free()


def test_power_of_two_pattern_through_caller_supplied_lists():
    # not banded (depends on the flattened distance): the caller builds the lists
    N, block, D = 3000, 128, 64
    print("power-of-two lists", flush=True)
    bitmap = op.block_bitmap(lambda rows: op.power_of_two_rows(N, rows, local=64), N, block)
    row_ptr, col_idx = om.block_lists(bitmap)
    mask = rb.radial_mask_from_csr(N, block, row_ptr, col_idx, rb.RADIAL_MASK_TRANSPOSE)
    q, k, v, do = (_randn_bf16((1, 1, N, D), 81 + i) for i in range(4))
    got = _attention_all(q, k, v, do, mask, 0.125)
    vis = np.repeat(np.repeat(bitmap, block, axis=0), block, axis=1)[:N, :N]
    _check_against(vis, q, k, v, do, 0.125, got)
    mask.free()
