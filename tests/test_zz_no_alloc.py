"""radial_attn_bwd_static (the backward for callers that cannot allocate) against radial_attn_bwd,
through the C ABI, on two calls in a row, the second with a smaller input (run with -m gpu).

The two entry points share their kernels and differ only in where the per-row sums live (the
caller's workspace / the library's own device array), so the gradients must be identical bit
for bit; radial_attn_bwd itself is compared with the float64 oracle in test_gpu_bwd.py, and
the first case here repeats that comparison for the new entry point."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import attention as oa
from oracle import build as obuild
from paper_2506_19852_amd import binding as rb

from util import assert_close

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _randn_bf16(shape, seed):
    g = torch.Generator(device="cpu").manual_seed(seed)
    return torch.randn(shape, generator=g).to(torch.bfloat16).to(DEV)


def _case(f, s, block, D, B, H, seed):
    N = f * s
    q, k, v, do = (_randn_bf16((B, H, N, D), seed + i) for i in range(4))
    scale = 1.0 / np.sqrt(D)
    mask = rb.radial_mask_build(f, s, block, 1, rb.RADIAL_MASK_TRANSPOSE)
    out = torch.empty_like(q)
    lse = torch.empty((B, H, N), dtype=torch.float32, device=DEV)
    rb.radial_attn_fwd(q, k, v, out, lse, mask, scale)
    return dict(q=q, k=k, v=v, do=do, out=out, lse=lse, mask=mask, scale=scale, shape=(f, s, block, D, B, H))


def _existing(c):
    B, H, N, D = c["q"].shape
    ws = torch.empty(rb.radial_attn_bwd_workspace(B, H, N, D, c["mask"]), dtype=torch.uint8, device=DEV)
    g = [torch.full_like(c["q"], float("nan")) for _ in range(3)]
    rb.radial_attn_bwd(c["q"], c["k"], c["v"], c["out"], c["do"], c["lse"], *g, c["mask"], c["scale"], ws)
    torch.cuda.synchronize()
    return g


def _static(c):
    g = [torch.full_like(c["q"], float("nan")) for _ in range(3)]
    rb.radial_attn_bwd_static(c["q"], c["k"], c["v"], c["out"], c["do"], c["lse"], *g, c["mask"], c["scale"])
    torch.cuda.synchronize()
    return g


def test_two_calls_in_a_row_second_smaller():
    big = _case(9, 300, 128, 128, 1, 3, 700)     # N = 2700: 22 blocks, ragged tail, blocks straddle frames
    small = _case(5, 200, 64, 64, 2, 1, 800)     # N = 1000, other block size and head dimension
    want_big, want_small = _existing(big), _existing(small)
    for c, want, name in ((big, want_big, "first call"), (small, want_small, "second, smaller call")):
        print(f"radial_attn_bwd_static {name}: f,s,block,D,B,H = {c['shape']}", flush=True)
        got = _static(c)
        for g, w, nm in zip(got, want, ("dQ", "dK", "dV")):
            assert torch.equal(g.view(torch.int16), w.view(torch.int16)), f"{name}: {nm} differs from radial_attn_bwd"
    # and against the oracle, one head of the first case
    f, s, block, D, B, H = big["shape"]
    bitmap, _ = obuild.mask_scan(f, s, block, 1)
    n = f * s
    vis = np.repeat(np.repeat(bitmap, block, axis=0), block, axis=1)[:n, :n]
    got = _static(big)
    q, k, v, do = (big[t][0, 1].float().cpu().numpy() for t in ("q", "k", "v", "do"))
    ref = oa.attention_bwd_rows(q, k, v, vis, big["scale"], do)[:3]
    for g, w, nm in zip(got, ref, ("dQ", "dK", "dV")):
        assert_close(g[0, 1].float().cpu().numpy(), w, f"static backward vs oracle {nm}")
    big["mask"].free()
    small["mask"].free()


def test_too_large_is_rejected_without_a_launch():
    lib = rb.load()
    limit = 24 << 20
    # B*H*N floats beyond the array: one head of 128 tokens times enough (batch, head) pairs
    f, s, block, D = 1, 128, 128, 64
    mask = rb.radial_mask_build(f, s, block, 1, rb.RADIAL_MASK_TRANSPOSE)
    B, H = 1, limit // 4 // 128 + 1
    t = rb.radial_tensor(ctypes.c_void_p(256), 0, 0, 64)   # never dereferenced: the size check comes first
    rc = lib.radial_attn_bwd_static(B, H, 128, D, t, t, t, t, t, ctypes.c_void_p(256), t, t, t, mask.handle,
                                    ctypes.c_float(0.125), None)
    assert rc == -5 and "scratch" in rb.radial_last_error()
    mask.free()
