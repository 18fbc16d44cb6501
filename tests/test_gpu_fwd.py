"""GPU block-sparse attention forward vs the float64 oracle (run with -m gpu)."""
import numpy as np
import pytest
import torch

from oracle import build as obuild
from oracle import mask as om
from paper_2506_19852_amd import binding as rb
from paper_2506_19852_amd import workloads as wl

from util import assert_close, oracle_fwd_block, sample_qblocks

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _run_fwd(q, k, v, mask, scale, want_lse=True):
    out = torch.full_like(q, float("nan"))
    lse = torch.full(q.shape[:3], float("nan"), dtype=torch.float32, device=q.device) if want_lse else None
    rb.radial_attn_fwd(q, k, v, out, lse, mask, scale)
    torch.cuda.synchronize()
    return out, lse


def _check_blocks(out, lse, q, k, v, bitmap_rows, qblocks, block, scale, head_pairs, what):
    """Compares the query blocks `qblocks` of the (b, h) pairs in head_pairs with the oracle."""
    worst = 0.0
    for (b, h) in head_pairs:
        qh, kh, vh = (t[b, h].float().cpu().numpy() for t in (q, k, v))
        oh = out[b, h].float().cpu().numpy()
        lh = lse[b, h].cpu().numpy() if lse is not None else None
        for qb, row in zip(qblocks, bitmap_rows):
            ref_o, ref_l = oracle_fwd_block(qh, kh, vh, row, qb, block, scale)
            r0 = qb * block
            err, _ = assert_close(oh[r0:r0 + ref_o.shape[0]], ref_o, f"{what} b{b} h{h} qb{qb} O")
            worst = max(worst, err)
            if lh is not None:
                got_l = lh[r0:r0 + ref_l.shape[0]]
                fin = np.isfinite(ref_l)
                assert np.array_equal(np.isneginf(got_l), ~fin)
                assert np.allclose(got_l[fin], ref_l[fin], rtol=1e-4, atol=1e-4), f"{what} b{b} h{h} qb{qb} LSE"
    return worst


def _randn_bf16(shape, seed, scale=1.0):
    g = torch.Generator(device="cpu").manual_seed(seed)
    return (torch.randn(shape, generator=g) * scale).to(torch.bfloat16).to(DEV)


# ---- config 1: every element, radial and dense ------------------------------------------------

def test_cfg1_every_element():
    w = wl.WORKLOADS["cfg1_tiny"]
    print("fwd cfg1", flush=True)
    x = wl.make_inputs(w, DEV)
    f, s, block = w.frames, w.tokens_per_frame, w.block
    for kind in ("radial", "dense"):
        if kind == "radial":
            mask = rb.radial_mask_build(f, s, block, 1)
            bitmap, _ = obuild.mask_scan(f, s, block, 1)
        else:
            mask = rb.radial_mask_build_dense(w.N, block)
            bitmap = np.ones((w.N // block, w.N // block), dtype=bool)
        out, lse = _run_fwd(x["q"], x["k"], x["v"], mask, w.scale)
        nb = bitmap.shape[0]
        _check_blocks(out, lse, x["q"], x["k"], x["v"], bitmap, range(nb), block, w.scale,
                      [(0, h) for h in range(w.H)], f"cfg1 {kind}")
        mask.free()


# ---- small shapes: ragged tails, straddling blocks, both head dims, strides, peaked softmax ------

@pytest.mark.parametrize("f,s,block,D,B,H,sink,qscale", [
    (5, 200, 128, 128, 1, 2, 1, 1.0),      # N = 1000: ragged last block, blocks straddle frames
    (5, 200, 64, 64, 2, 1, 0, 1.0),
    (3, 333, 128, 64, 1, 2, 1, 1.0),       # N = 999
    (7, 100, 64, 128, 1, 1, 2, 1.0),
    (9, 150, 128, 128, 1, 2, 1, 6.0),      # peaked rows: exercises the running-max rescale
    (40, 24, 128, 128, 1, 1, 1, 1.0),      # several frames inside one block
    (1, 65, 64, 64, 1, 1, 1, 1.0),         # two blocks, second holds one token
    (1, 1, 128, 128, 1, 1, 1, 1.0),        # one token
])
def test_small_shapes(f, s, block, D, B, H, sink, qscale):
    print(f"fwd small f={f} s={s} block={block} D={D} B={B} H={H} sink={sink} qscale={qscale}", flush=True)
    N = f * s
    q = _randn_bf16((B, H, N, D), 11, qscale)
    k = _randn_bf16((B, H, N, D), 12)
    v = _randn_bf16((B, H, N, D), 13)
    scale = 1.0 / np.sqrt(D)
    mask = rb.radial_mask_build(f, s, block, sink)
    bitmap, _ = obuild.mask_scan(f, s, block, sink)
    out, lse = _run_fwd(q, k, v, mask, scale)
    pairs = [(b, h) for b in range(B) for h in range(H)]
    _check_blocks(out, lse, q, k, v, bitmap, range(bitmap.shape[0]), block, scale, pairs, "small")
    # without LSE
    out2, _ = _run_fwd(q, k, v, mask, scale, want_lse=False)
    assert torch.equal(out, out2)
    mask.free()


def test_strided_layout_and_user_list():
    # tensors stored [B, N, H, D] (token-major) and handed over as [B, H, N, D] views
    B, H, N, D, block = 2, 3, 700, 128, 128
    print("fwd strided + user list", flush=True)
    base = [_randn_bf16((B, N, H, D), 20 + i) for i in range(3)]
    q, k, v = (t.permute(0, 2, 1, 3) for t in base)
    nb = -(-N // block)
    rng = np.random.default_rng(5)
    bitmap = rng.random((nb, nb)) < 0.5
    bitmap[2] = False                                  # an empty row: O = 0, LSE = -inf
    row_ptr, col_idx = om.block_lists(bitmap)
    mask = rb.radial_mask_from_csr(N, block, row_ptr, col_idx)
    out_base = torch.full((B, N, H, D), float("nan"), dtype=torch.bfloat16, device=DEV)
    out = out_base.permute(0, 2, 1, 3)
    lse = torch.full((B, H, N), float("nan"), dtype=torch.float32, device=DEV)
    rb.radial_attn_fwd(q, k, v, out, lse, mask, 0.11)
    torch.cuda.synchronize()
    pairs = [(b, h) for b in range(B) for h in range(H)]
    _check_blocks(out, lse, q, k, v, bitmap, range(nb), block, 0.11, pairs, "strided")
    assert (out[:, :, 2 * block:3 * block] == 0).all() and torch.isneginf(lse[:, :, 2 * block:3 * block]).all()
    mask.free()


def test_row_maximum_spans_all_keys_of_a_stage():
    # Keys whose index has bit 2 set score +L, the others -L: the running maximum has to come
    # from every key of a 64-key stage, or exp() of the difference overflows.
    N, D, block = 512, 128, 128
    print("fwd row maximum", flush=True)
    g = torch.Generator(device="cpu").manual_seed(77)
    u = torch.randn(D, generator=g)
    u = u / u.norm()
    q = (u[None, :] * 16.0 + 0.05 * torch.randn((N, D), generator=g)).to(torch.bfloat16)
    sign = torch.where((torch.arange(N) & 4) != 0, 1.0, -1.0)
    k = (sign[:, None] * u[None, :] * 16.0 + 0.05 * torch.randn((N, D), generator=g)).to(torch.bfloat16)
    v = torch.randn((N, D), generator=g).to(torch.bfloat16)
    q, k, v = (t.view(1, 1, N, D).to(DEV) for t in (q, k, v))
    scale = 0.5                                       # logits about +-128
    mask = rb.radial_mask_build_dense(N, block)
    out, lse = _run_fwd(q, k, v, mask, scale)
    bitmap = np.ones((N // block, N // block), dtype=bool)
    _check_blocks(out, lse, q, k, v, bitmap, range(N // block), block, scale, [(0, 0)], "rowmax")
    mask.free()


def test_argument_errors():
    q = _randn_bf16((1, 1, 256, 64), 1)
    mask = rb.radial_mask_build(2, 128, 64, 1)
    out = torch.empty_like(q)
    bad = torch.empty((1, 1, 256, 96), dtype=torch.bfloat16, device=DEV)
    with pytest.raises(rb.RadialError) as e:
        rb.radial_attn_fwd(bad, bad, bad, torch.empty_like(bad), None, mask, 0.1)
    assert e.value.code == -4
    q2 = _randn_bf16((1, 1, 320, 64), 1)
    with pytest.raises(rb.RadialError) as e:
        rb.radial_attn_fwd(q2, q2, q2, torch.empty_like(q2), None, mask, 0.1)
    assert e.value.code == -5
    with pytest.raises(rb.RadialError) as e:
        rb.radial_attn_fwd(q, q, q, out, None, mask, float("nan"))
    assert e.value.code == -1
    mis = torch.empty(256 * 64 + 8, dtype=torch.bfloat16, device=DEV)[4:4 + 256 * 64].view(1, 1, 256, 64)
    with pytest.raises(rb.RadialError) as e:
        rb.radial_attn_fwd(mis, q, q, out, None, mask, 0.1)
    assert e.value.code == -5
    mask.free()


# ---- full-size workloads, in the launch configuration the benchmark times ---------------------------

@pytest.mark.parametrize("name,heads,nsample", [
    ("cfg2_wan480p", (0, 39), None),               # two complete heads
    ("cfg3_hunyuan720p", (0, 23), 64),
    ("cfg4_hunyuan720p_4x", (5,), 64),
    ("cfg5_wan480p_4x_bwd", (17,), 48),
])
def test_workload_forward(name, heads, nsample):
    w = wl.WORKLOADS[name]
    print(f"fwd workload {name}", flush=True)
    f, s, block = w.frames, w.tokens_per_frame, w.block
    x = {nm: wl.make_tensor(w, nm, DEV) for nm in ("q", "k", "v")}
    mask = rb.radial_mask_build(f, s, block, 1)
    row_ptr, _ = rb.radial_mask_copy_to_host(mask)
    nb = row_ptr.size - 1
    out, lse = _run_fwd(x["q"], x["k"], x["v"], mask, w.scale)
    qblocks = list(range(nb)) if nsample is None else sample_qblocks(nb, np.diff(row_ptr), s, block, nsample, w.seed)
    rows = []
    for qb in qblocks:                                     # oracle lists of the sampled blocks
        bm, _ = obuild.mask_scan(f, s, block, 1, qb, qb + 1)
        rows.append(bm[0])
    worst = _check_blocks(out, lse, x["q"], x["k"], x["v"], rows, qblocks, block, w.scale,
                          [(0, h) for h in heads], name)
    print(f"{name}: {len(qblocks)} query blocks x {len(heads)} heads checked, max |err| {worst:.3e}", flush=True)
    # properties that hold for every row: finite output, |O| bounded by max |V| of the head
    of = out.float()
    assert torch.isfinite(of).all() and torch.isfinite(lse).all()
    assert (of.abs().amax(dim=(2, 3)) <= x["v"].float().abs().amax(dim=(2, 3)) + 1e-3).all()
    mask.free()


# ---- the long end of the complexity curve --------------------------------------------------------

@pytest.mark.parametrize("frames,n_sample,n_dense", [(257, 10, 2), (509, 6, 1)])
def test_long_video_sampled_blocks(frames, n_sample, n_dense):
    """The long end of the forward-time curve at the 720p geometry, one head: 257 frames
    (N = 925 200, the last point of the benchmark's sweep) and 509 frames (N = 1 832 400, the length
    at which Fig. 2 of the paper quotes its attention-compute saving).  The lists of sampled query
    blocks bit-exact against the oracle's scan, their outputs against the oracle, radial list and
    all-ones list."""
    import dataclasses
    base = wl.WORKLOADS["cfg3_hunyuan720p"]
    w = dataclasses.replace(base, name=f"hunyuan720p_f{frames}", frames=frames, H=1)
    f, s, block = w.frames, w.tokens_per_frame, w.block
    print(f"fwd long video f={f} N={w.N}", flush=True)
    x = wl.make_inputs(w, DEV)
    mask = rb.radial_mask_build(f, s, block, 1)
    row_ptr, col_idx = rb.radial_mask_copy_to_host(mask)
    nb = row_ptr.size - 1
    assert nb == -(-w.N // block) and w.N % block != 0                     # ragged last block
    qblocks = sample_qblocks(nb, np.diff(row_ptr), s, block, n_sample, w.seed)
    rows = []
    for qb in qblocks:
        bm, _ = obuild.mask_scan(f, s, block, 1, qb, qb + 1)
        assert np.array_equal(np.flatnonzero(bm[0]), col_idx[row_ptr[qb]:row_ptr[qb + 1]]), f"list of query block {qb}"
        rows.append(bm[0])
    out, lse = _run_fwd(x["q"], x["k"], x["v"], mask, w.scale)
    worst = _check_blocks(out, lse, x["q"], x["k"], x["v"], rows, qblocks, block, w.scale, [(0, 0)], f"{frames} frames radial")
    print(f"{frames} frames, radial list: {len(qblocks)} query blocks (lists of {min(r.sum() for r in rows)} to "
          f"{max(r.sum() for r in rows)} blocks of {nb}), max |err| {worst:.2e}", flush=True)
    mask.free()
    dense = rb.radial_mask_build_dense(w.N, block)
    out, lse = _run_fwd(x["q"], x["k"], x["v"], dense, w.scale)
    ones = np.ones(nb, dtype=bool)
    picks = [nb - 1, qblocks[1]][:n_dense]
    worst = _check_blocks(out, lse, x["q"], x["k"], x["v"], [ones] * len(picks), picks, block, w.scale, [(0, 0)],
                          f"{frames} frames dense")
    print(f"{frames} frames, all-ones list: {len(picks)} query blocks, max |err| {worst:.2e}", flush=True)
    dense.free()
