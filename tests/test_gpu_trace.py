"""GPU tests of the measurement entry points: the traced forward and the MFMA probe."""
import numpy as np
import pytest
import torch

from paper_2506_19852_amd import binding as rb

pytestmark = pytest.mark.gpu


def test_traced_forward_matches_the_plain_call_and_fills_one_record_per_workgroup():
    f, s, block, B, H, D = 6, 200, 128, 1, 3, 128
    N = f * s
    g = torch.Generator(device="cpu").manual_seed(11)
    q, k, v = (torch.randn((B, H, N, D), generator=g).to(torch.bfloat16).cuda() for _ in range(3))
    m = rb.radial_mask_build(f, s, block, 1, 0)
    ref, out = torch.empty_like(q), torch.empty_like(q)
    lse_ref = torch.empty((B, H, N), dtype=torch.float32, device="cuda")
    lse = torch.empty_like(lse_ref)
    rb.radial_attn_fwd(q, k, v, ref, lse_ref, m, D ** -0.5)
    n_rec = rb.radial_attn_fwd_trace_records(B, H, m)
    n_blocks = (N + block - 1) // block
    assert n_rec >= B * H * n_blocks and n_rec % 8 == 0
    trace = torch.zeros((n_rec, 3), dtype=torch.int64, device="cuda")
    rb.radial_attn_fwd_trace(q, k, v, out, lse, m, D ** -0.5, trace)
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), ref.view(torch.int16))
    assert torch.equal(lse, lse_ref)
    t = trace.cpu().numpy()
    used = t[:, 1] != 0
    assert int(used.sum()) == B * H * n_blocks          # one record per (head, query block)
    assert np.all(t[used, 1] >= t[used, 0]) and np.all(t[used, 0] > 0)
    assert np.all(t[~used] == 0)
    assert np.all(((t[used, 2] >> 32) & 0xF) < 8)
    # too few records: refused before any launch
    small = torch.zeros((n_rec - 1, 3), dtype=torch.int64, device="cuda")
    with pytest.raises(rb.RadialError) as e:
        rb.radial_attn_fwd_trace(q, k, v, out, lse, m, D ** -0.5, small)
    assert e.value.code == -5          # RADIAL_ESHAPE
    m.free()


def test_mfma_probe_runs_and_counts_its_operations():
    flops = rb.radial_probe_mfma_bf16(100)
    torch.cuda.synchronize()
    assert flops == 256 * 8 * 16 * 100 * 4 * (2 * 32 * 32 * 16)
    with pytest.raises(rb.RadialError):
        rb.radial_probe_mfma_bf16(6)
