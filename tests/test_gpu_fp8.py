"""GPU tests of the 8-bit scores: the quantiser bit-exact against the oracle's, and the forward
against the float64 oracle run on the dequantised Q and K (same mask, same V)."""
import numpy as np
import pytest
import torch

from oracle import attention as oa
from oracle import build as obuild
from oracle import quant
from paper_2506_19852_amd import binding as rb

pytestmark = pytest.mark.gpu


def _bf16(shape, seed, scale=1.0):
    g = torch.Generator(device="cpu").manual_seed(seed)
    return (torch.randn(shape, generator=g) * scale).to(torch.bfloat16)


@pytest.mark.parametrize("N, D, block", [(300, 128, 128), (1000, 64, 64), (257, 128, 128)])
def test_quantiser_matches_the_oracle_bit_for_bit(N, D, block):
    B, H = 2, 3
    x = _bf16((B, H, N, D), 3)
    x[0, 1, 128:256] = 0            # an all-zero block
    x[1, 2, 5, 7] = 37.5            # an outlier that sets its block's scale
    nb = (N + block - 1) // block
    codes = torch.empty((B, H, N, D), dtype=torch.uint8, device="cuda")
    scales = torch.empty((B, H, nb), dtype=torch.float32, device="cuda")
    rb.radial_quantize_fp8(x.cuda(), block, codes, scales)
    torch.cuda.synchronize()
    for b in range(B):
        for h in range(H):
            want_c, want_s = quant.quantize_blocks(x[b, h].float().numpy(), block)
            assert np.array_equal(scales[b, h].cpu().numpy(), want_s), (b, h)
            assert np.array_equal(codes[b, h].cpu().numpy(), want_c), (b, h)


def test_quantiser_reads_strided_tensors():
    B, H, N, D = 1, 2, 200, 128
    big = _bf16((B, N, H, D + 64), 5).cuda()
    x = big[..., :D].permute(0, 2, 1, 3)            # [B, H, N, D] view with padded rows
    codes = torch.empty((B, H, N, D), dtype=torch.uint8, device="cuda")
    scales = torch.empty((B, H, 2), dtype=torch.float32, device="cuda")
    rb.radial_quantize_fp8(x, 128, codes, scales)
    torch.cuda.synchronize()
    for h in range(H):
        want_c, want_s = quant.quantize_blocks(x[0, h].float().cpu().numpy(), 128)
        assert np.array_equal(codes[0, h].cpu().numpy(), want_c) and np.array_equal(scales[0, h].cpu().numpy(), want_s)


@pytest.mark.parametrize("f, s, sink, qscale", [(6, 200, 1, 1.0), (5, 333, 0, 4.0), (3, 128, 1, 1.0), (1, 50, 1, 1.0),
                                                  (40, 3, 0, 1.0), (2, 300, 5, 0.25)])
def test_forward_with_8bit_scores_matches_the_oracle_on_dequantised_inputs(f, s, sink, qscale):
    B, H, D, block = 1, 2, 128, 128
    N = f * s
    q, k, v = _bf16((B, H, N, D), 21, qscale), _bf16((B, H, N, D), 22), _bf16((B, H, N, D), 23)
    nb = (N + block - 1) // block
    m = rb.radial_mask_build(f, s, block, sink, 0)
    row_ptr, col_idx = rb.radial_mask_copy_to_host(m)
    qc = torch.empty((B, H, N, D), dtype=torch.uint8, device="cuda")
    kc = torch.empty_like(qc)
    qs = torch.empty((B, H, nb), dtype=torch.float32, device="cuda")
    ks = torch.empty_like(qs)
    rb.radial_quantize_fp8(q.cuda(), block, qc, qs)
    rb.radial_quantize_fp8(k.cuda(), block, kc, ks)
    out = torch.empty((B, H, N, D), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty((B, H, N), dtype=torch.float32, device="cuda")
    scale = D ** -0.5
    rb.radial_attn_fwd_fp8(qc, qs, kc, ks, v.cuda(), out, lse, m, scale)
    torch.cuda.synchronize()
    got_o, got_l = out.float().cpu().numpy(), lse.cpu().numpy()
    bitmap = obuild.mask_scan(f, s, block, sink)[0]        # the oracle's own block mask
    for h in range(H):
        qd = quant.dequantize_blocks(*quant.quantize_blocks(q[0, h].float().numpy(), block), block)
        kd = quant.dequantize_blocks(*quant.quantize_blocks(k[0, h].float().numpy(), block), block)
        vv = v[0, h].float().numpy()
        for qb in range(nb):
            cols = np.nonzero(bitmap[qb])[0]
            assert np.array_equal(cols, col_idx[row_ptr[qb]:row_ptr[qb + 1]])
            keys = (cols[:, None] * block + np.arange(block)[None, :]).ravel()
            keys = keys[keys < N]
            rows = np.arange(qb * block, min(N, (qb + 1) * block))
            ref_o, ref_l = oa.attention_rows_keyset(qd[rows], kd, vv, keys, scale)[:2]
            err = np.abs(got_o[0, h, rows] - ref_o)
            assert np.all(err <= 1e-2 + 1e-2 * np.abs(ref_o)), (h, qb, err.max())
            assert err.max() <= 2e-2 * max(np.abs(ref_o).max(), 1e-6) + 1e-3, (h, qb, err.max())
            assert np.allclose(got_l[0, h, rows], ref_l, rtol=1e-4, atol=1e-4), (h, qb)
    m.free()


def test_8bit_forward_refuses_what_it_does_not_support():
    B, H, N, D = 1, 1, 256, 128
    m = rb.radial_mask_build(2, 128, 128, 1, rb.RADIAL_MASK_TOKEN_EXACT)
    qc = torch.zeros((B, H, N, D), dtype=torch.uint8, device="cuda")
    qs = torch.ones((B, H, 2), dtype=torch.float32, device="cuda")
    v = torch.zeros((B, H, N, D), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(rb.RadialError) as e:
        rb.radial_attn_fwd_fp8(qc, qs, qc, qs, v, torch.empty_like(v), None, m, 0.1)
    assert e.value.code == -4          # RADIAL_EUNSUPPORTED
    m.free()
    # codes quantised per 64 tokens do not fit a mask of 128-token blocks
    m = rb.radial_mask_build(2, 128, 128, 1, 0)
    qs64 = torch.ones((B, H, 4), dtype=torch.float32, device="cuda")
    with pytest.raises(rb.RadialError) as e:
        rb.radial_attn_fwd_fp8(qc, qs64, qc, qs64, v, torch.empty_like(v), None, m, 0.1, code_block=64)
    assert e.value.code == -5          # RADIAL_ESHAPE
    m.free()


def test_8bit_forward_at_the_benchmark_workload_sampled_blocks():
    """cfg3 in the launch configuration `bench.py --fp8-scores` times: sampled query blocks of two heads."""
    from paper_2506_19852_amd import workloads as wl
    from util import assert_close, oracle_fwd_block, sample_qblocks
    w = wl.WORKLOADS["cfg3_hunyuan720p"]
    f, s, block = w.frames, w.tokens_per_frame, w.block
    x = {nm: wl.make_tensor(w, nm, "cuda:0") for nm in ("q", "k", "v")}
    nb = (w.N + block - 1) // block
    m = rb.radial_mask_build(f, s, block, 1, 0)
    row_ptr, _ = rb.radial_mask_copy_to_host(m)
    qc = torch.empty(x["q"].shape, dtype=torch.uint8, device="cuda")
    kc = torch.empty_like(qc)
    qs = torch.empty((w.B, w.H, nb), dtype=torch.float32, device="cuda")
    ks = torch.empty_like(qs)
    rb.radial_quantize_fp8(x["q"], block, qc, qs)
    rb.radial_quantize_fp8(x["k"], block, kc, ks)
    out = torch.empty_like(x["q"])
    lse = torch.empty((w.B, w.H, w.N), dtype=torch.float32, device="cuda")
    rb.radial_attn_fwd_fp8(qc, qs, kc, ks, x["v"], out, lse, m, w.scale)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all() and torch.isfinite(lse).all()
    qblocks = sample_qblocks(nb, np.diff(row_ptr), s, block, 24, w.seed)
    worst = 0.0
    for h in (0, 23):
        qn, kn, vn = (x[nm][0, h].float().cpu().numpy() for nm in ("q", "k", "v"))
        qcodes, qscales = quant.quantize_blocks(qn, block)
        kcodes, kscales = quant.quantize_blocks(kn, block)
        assert np.array_equal(qc[0, h].cpu().numpy(), qcodes) and np.array_equal(ks[0, h].cpu().numpy(), kscales)
        qd, kd = quant.dequantize_blocks(qcodes, qscales, block), quant.dequantize_blocks(kcodes, kscales, block)
        oh, lh = out[0, h].float().cpu().numpy(), lse[0, h].cpu().numpy()
        for qb in qblocks:
            bm, _ = obuild.mask_scan(f, s, block, 1, qb, qb + 1)
            ref_o, ref_l = oracle_fwd_block(qd, kd, vn, bm[0], qb, block, w.scale)
            r0 = qb * block
            err, _ = assert_close(oh[r0:r0 + ref_o.shape[0]], ref_o, f"fp8 cfg3 h{h} qb{qb} O")
            assert np.allclose(lh[r0:r0 + ref_o.shape[0]], ref_l, rtol=1e-4, atol=1e-4), f"fp8 cfg3 h{h} qb{qb} LSE"
            worst = max(worst, err)
    print(f"fp8 cfg3: {len(qblocks)} query blocks x 2 heads checked, max |err| {worst:.3e}", flush=True)
    # What the quantisation itself costs: the same blocks against the bf16 path and against the
    # oracle on the ORIGINAL q, k (reported; the 8-bit scores are an optional reduced-precision extra).
    out16 = torch.empty_like(x["q"])
    rb.radial_attn_fwd(x["q"], x["k"], x["v"], out16, None, m, w.scale)
    torch.cuda.synchronize()
    d_bf16, d_exact, ref_max = 0.0, 0.0, 0.0
    for h in (0, 23):
        qn, kn, vn = (x[nm][0, h].float().cpu().numpy() for nm in ("q", "k", "v"))
        for qb in qblocks[:8]:
            bm, _ = obuild.mask_scan(f, s, block, 1, qb, qb + 1)
            ref_o, _ = oracle_fwd_block(qn, kn, vn, bm[0], qb, block, w.scale)
            r0, r1 = qb * block, qb * block + ref_o.shape[0]
            o8, o16 = out[0, h, r0:r1].float().cpu().numpy(), out16[0, h, r0:r1].float().cpu().numpy()
            d_bf16 = max(d_bf16, float(np.abs(o8 - o16).max()))
            d_exact = max(d_exact, float(np.abs(o8 - ref_o).max()))
            ref_max = max(ref_max, float(np.abs(ref_o).max()))
    print(f"fp8 cfg3: max |O_fp8 - O_bf16| = {d_bf16:.3e}, max |O_fp8 - oracle(original q,k)| = {d_exact:.3e}, "
          f"max |O| = {ref_max:.3e}", flush=True)
    assert d_exact <= 1e-2 + 1e-2 * ref_max        # the benchmark spec's absolute term still holds at this workload
    m.free()
