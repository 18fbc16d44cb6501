#!/usr/bin/env python3
"""Benchmark of the radial-attention hot path on one MI355X.

A step = the radial mask build + one block-sparse attention forward over the whole
[B, H, N, D] workload (plus the backward for the forward+backward workload).  Inputs are
synthetic and resident in HBM before the timed region.  Prints one JSON line: effective
TFLOP/s on computed blocks, the kernel's fraction of the bf16 MFMA peak, the dense baseline
(same kernel, all-ones list) and the CPU oracle timed on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 MFMA

PROFILES = os.path.join(ROOT, "profiles")
# Sources of the attention kernels: a counter summary under profiles/ names the files it depends on
# and their digest, so that a summary taken on other kernel code is recognised whatever the speed
# of the box it was taken on.
FWD_KERNEL_SOURCES = ("radial_attn_fwd.hip", "radial_attn_fwd_kernel.h", "radial_tile.h", "radial_internal.h")
BWD_KERNEL_SOURCES = FWD_KERNEL_SOURCES + ("radial_attn_bwd.hip",)


def kernel_source_digest(names=BWD_KERNEL_SOURCES) -> str:
    """First 16 hex digits of the SHA-256 over the named source files of the attention kernels."""
    import hashlib
    h = hashlib.sha256()
    for name in names:
        with open(os.path.join(ROOT, "paper_2506_19852_amd", "csrc", os.path.basename(name)), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def traffic_from_profile(workload: str, timed_kernel_ms: float, copy_bytes: float):
    """HBM-side bytes per forward launch from the committed rocprofv3 counter summary of this
    workload (profiles/fwd_<workload>.txt): FETCH_SIZE and WRITE_SIZE of the radial-list launches
    (KiB per dispatch), each scaled by what the same counter read for a streaming copy of known
    size in the same run.  Returns (bytes or None, source): None when there is no summary or
    when the counters were not taken on the kernel that is running: the summary names the digest
    of the kernel source files it was taken on, which must equal their digest now (boxes differ
    by several per cent in speed, the sources do not); a summary without that line counts only
    if its kernel time is within 3 % of the one timed now."""
    import re
    name = {"cfg5_wan480p_4x_bwd": "fwd_bwd_cfg5_wan480p_4x.txt"}.get(workload, f"fwd_{workload}.txt")
    path = os.path.join(PROFILES, name)
    src = {"file": os.path.relpath(path, ROOT), "kernel_ms_at_capture": None}
    try:
        text = open(path).read()
    except OSError:
        return None, dict(src, note="no counter summary for this workload")
    def grab(pattern):
        m = re.search(pattern, text, flags=re.M)
        return float(m.group(1)) if m else None
    ms = grab(r"^radial_fwd\w*<[^>]*> radial list\s+\d+\s+([0-9.]+)")
    fetch = grab(r"radial list\s+FETCH_SIZE\s+avg/launch ([0-9.e+]+)")
    write = grab(r"radial list\s+WRITE_SIZE\s+avg/launch ([0-9.e+]+)")
    cp_fetch = grab(r"copy probe[^\n]*FETCH_SIZE ([0-9.e+]+) KiB")
    cp_write = grab(r"copy probe[^\n]*WRITE_SIZE ([0-9.e+]+) KiB")
    src["kernel_ms_at_capture"] = ms
    if None in (ms, fetch, write, cp_fetch, cp_write):
        return None, dict(src, note="summary lacks a figure")
    m = re.search(r"^# kernel sources at capture \([^)]*, of ([\w. ]+)\): ([0-9a-f]{16})\s*$", text, flags=re.M)
    if m:
        src["kernel_sources_at_capture"] = m.group(2)
        try:
            same = m.group(2) == kernel_source_digest(m.group(1).split())
        except OSError:
            same = False
        if not same:
            return None, dict(src, note="the kernel sources have changed since the capture")
        if abs(ms - timed_kernel_ms) > 0.15 * timed_kernel_ms:
            return None, dict(src, note="kernel time differs from the captured one by more than 15 %")
    elif abs(ms - timed_kernel_ms) > 0.03 * timed_kernel_ms:
        return None, dict(src, note="kernel time differs from the captured one by more than 3 %")
    known_kib = copy_bytes / 1024.0
    src["fetch_scale"], src["write_scale"] = round(known_kib / cp_fetch, 3), round(known_kib / cp_write, 3)
    return (fetch * known_kib / cp_fetch + write * known_kib / cp_write) * 1024.0, src


def effective_flops(row_ptr, col_idx, n_tokens, block, D, heads):
    """4*D*sum over listed pairs of rows(qb)*cols(kb): both products, real tokens only."""
    import numpy as np
    nb = row_ptr.size - 1
    size = np.full(nb, block, dtype=np.int64)
    size[-1] = n_tokens - (nb - 1) * block
    rows = np.repeat(size, np.diff(row_ptr).astype(np.int64))
    pairs = int((rows * size[col_idx]).sum())
    return 4 * D * pairs * heads


def cpu_baseline(w, x, row_ptr, col_idx, gpu_out=None, budget_s=12.0, max_blocks=None):
    """Times the CPU oracle (float64 numpy, as it stands) on query blocks of head 0 until the
    time budget is used; reports TFLOP/s with the same flop count as the GPU metric.  With
    gpu_out (the forward result, [B, H, N, D]) it also reports the largest absolute and relative
    error of the GPU result on the blocks the oracle computed."""
    import numpy as np
    from oracle import attention as oa
    q, k, v = (x[n][0, 0].float().cpu().numpy() for n in ("q", "k", "v"))
    got = gpu_out[0, 0].float().cpu().numpy() if gpu_out is not None else None
    nb = row_ptr.size - 1
    picks = np.random.default_rng(w.seed).permutation(nb)
    done, flops, t0 = 0, 0, time.perf_counter()
    max_abs, max_ref, max_rel = 0.0, 0.0, 0.0
    for qb in picks:
        cols = col_idx[row_ptr[qb]:row_ptr[qb + 1]]
        keys = (cols[:, None].astype(np.int64) * w.block + np.arange(w.block)[None, :]).ravel()
        keys = keys[keys < w.N]
        rows = np.arange(qb * w.block, min(w.N, (qb + 1) * w.block))
        ref = oa.attention_rows_keyset(q[rows], k, v, keys, w.scale)[0]
        flops += 4 * w.D * rows.size * keys.size
        done += 1
        if got is not None:
            err = np.abs(got[rows] - ref)
            max_abs = max(max_abs, float(err.max()))
            max_ref = max(max_ref, float(np.abs(ref).max()))
            max_rel = max(max_rel, float((err / (1e-2 + 1e-2 * np.abs(ref))).max()))
        if time.perf_counter() - t0 > budget_s or (max_blocks is not None and done >= max_blocks):
            break
    dt = time.perf_counter() - t0
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    total = effective_flops(row_ptr, col_idx, w.N, w.block, w.D, w.B * w.H)
    res = {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
           "sample": f"{done} of {nb} query blocks of head 0 ({w.name}), float64 numpy, {dt:.1f} s",
           "sampled_fraction_of_flops": flops / total, "extrapolated_full_forward_s": dt * total / flops}
    if got is not None:
        # err / (1e-2 + 1e-2 |ref|) <= 1 is the tolerance of the parity tests (1e-2 absolute + 1e-2 relative)
        res.update({"gpu_max_abs_err": max_abs, "gpu_max_abs_err_over_max_ref": max_abs / max_ref if max_ref else None,
                    "gpu_max_err_over_tolerance": max_rel * 1.0, "max_abs_ref": max_ref})
    return res


def load_balance(trace):
    """Busy time per compute unit and per XCD from the per-workgroup records of one traced forward launch."""
    import numpy as np
    used = trace[:, 1] != 0
    begin, end, where = trace[used, 0], trace[used, 1], trace[used, 2]
    span = float(end.max() - begin.min())                  # ticks of the 100 MHz clock
    xcc = (where >> 32) & 0xF
    cu = xcc * 256 + ((where >> 8) & 0xFF)                 # XCD, shader engine / array, compute unit
    busy = np.zeros(int(cu.max()) + 1)
    np.add.at(busy, cu, (end - begin).astype(np.float64))
    busy = busy[busy > 0]
    last = np.zeros(8)
    np.maximum.at(last, xcc, (end - begin.min()).astype(np.float64))
    # two workgroups are resident per compute unit, so a fully busy unit shows 2 x span
    occ = busy / (2.0 * span)
    return {"workgroups": int(used.sum()), "compute_units_seen": int(busy.size),
            "launch_span_ms": round(span / 1e5, 3),
            "cu_busy_frac_min_mean_max": [round(float(occ.min()), 3), round(float(occ.mean()), 3), round(float(occ.max()), 3)],
            "xcd_finish_frac_min_max": [round(float(last.min() / span), 3), round(float(last.max() / span), 3)],
            "xcd_is_workgroup_id_mod_8": round(float(np.mean(xcc == (np.nonzero(used)[0] & 7))), 4)}


def oracle_dq_error(w, x, grads, row_ptr, col_idx, qb):
    """Largest error of the GPU's dQ on query block qb of head 0 against the float64 oracle, as a
    multiple of the parity tolerance (1e-2 + 1e-2 |ref|).  Part of the CPU-baseline leg."""
    import numpy as np
    from oracle import attention as oa
    q, k, v, do = (x[n][0, 0].float().cpu().numpy() for n in ("q", "k", "v", "do"))
    cols = col_idx[row_ptr[qb]:row_ptr[qb + 1]]
    keys = (cols[:, None].astype(np.int64) * w.block + np.arange(w.block)[None, :]).ravel()
    keys = keys[keys < w.N]
    rows = np.arange(qb * w.block, min(w.N, (qb + 1) * w.block))
    ref = oa.attention_bwd_keyset(q[rows], k, v, keys, w.scale, do[rows])[0]
    err = np.abs(grads[0][0, 0, rows[0]:rows[-1] + 1].float().cpu().numpy() - ref)
    return {"dq_max_abs_err": float(err.max()), "dq_max_abs_ref": float(np.abs(ref).max()),
            "dq_max_err_over_tolerance": float((err / (1e-2 + 1e-2 * np.abs(ref))).max())}


def secondary_config(name, args, with_oracle):
    """One line of the `secondary` array: forward (and backward) kernel times of another
    workload, timed with events on the launch stream over a few launches, the same forward on
    the all-ones list, and -- inside the CPU-baseline leg -- the error of the GPU result on a
    sampled query block against the oracle."""
    import numpy as np
    import torch
    from paper_2506_19852_amd import binding as rb
    from paper_2506_19852_amd import workloads as wl
    w = wl.WORKLOADS[name]
    dev = "cuda:0"
    x = wl.make_inputs(w, dev)
    out = torch.empty_like(x["q"])
    lse = torch.empty((w.B, w.H, w.N), dtype=torch.float32, device=dev)
    m = rb.radial_mask_build(w.frames, w.tokens_per_frame, w.block, 1, rb.RADIAL_MASK_TRANSPOSE if w.backward else 0)
    row_ptr, col_idx = rb.radial_mask_copy_to_host(m)
    flops = effective_flops(row_ptr, col_idx, w.N, w.block, w.D, w.B * w.H)

    def timed(fn, launches):
        fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(launches):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1))
        return float(np.mean(ts))

    n = args.secondary_launches
    fwd_ms = timed(lambda: rb.radial_attn_fwd(x["q"], x["k"], x["v"], out, lse, m, w.scale), n)
    line = {"workload": w.name, "pass": "fwd+bwd" if w.backward else "fwd", "B": w.B, "H": w.H, "N": w.N, "D": w.D,
            "listed_block_pairs": int(row_ptr[-1]), "launches": n, "fwd_kernel_ms": round(fwd_ms, 3),
            "fwd_tflops": round(flops / fwd_ms / 1e9, 1), "fwd_frac": round(flops / fwd_ms / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4)}
    grads = None
    if w.backward:
        grads = [torch.empty_like(x["q"]) for _ in range(3)]
        ws = torch.empty(rb.radial_attn_bwd_workspace(w.B, w.H, w.N, w.D, m), dtype=torch.uint8, device=dev)
        bwd_ms = timed(lambda: rb.radial_attn_bwd(x["q"], x["k"], x["v"], out, x["do"], lse, *grads, m, w.scale, ws), n)
        # the gradient needs 5 products per listed pair against the forward's 2
        line.update({"bwd_kernels_ms": round(bwd_ms, 3), "bwd_tflops": round(2.5 * flops / bwd_ms / 1e9, 1),
                     "bwd_frac": round(2.5 * flops / bwd_ms / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4),
                     "fwd_bwd_tflops": round(3.5 * flops / (fwd_ms + bwd_ms) / 1e9, 1)})
    if with_oracle:
        base = cpu_baseline(w, x, row_ptr, col_idx, gpu_out=out, budget_s=4.0, max_blocks=2)
        line["oracle_check"] = {k2: base[k2] for k2 in ("sample", "gpu_max_abs_err", "max_abs_ref", "gpu_max_err_over_tolerance")}
        if w.backward:
            line["oracle_check"].update(oracle_dq_error(w, x, grads, row_ptr, col_idx, int(np.argmax(np.diff(row_ptr)))))
    m.free()
    dense = rb.radial_mask_build_dense(w.N, w.block)
    dptr, didx = rb.radial_mask_copy_to_host(dense)
    dense_flops = effective_flops(dptr, didx, w.N, w.block, w.D, w.B * w.H)
    dense_ms = timed(lambda: rb.radial_attn_fwd(x["q"], x["k"], x["v"], out, None, dense, w.scale), 1)
    dense.free()
    line.update({"dense_fwd_kernel_ms": round(dense_ms, 3), "dense_tflops": round(dense_flops / dense_ms / 1e9, 1),
                 "speedup_vs_dense": round(dense_ms / fwd_ms, 3), "block_ratio_dense_over_radial": round(dense_flops / flops, 3)})
    del x, out, lse, grads
    torch.cuda.empty_cache()
    return line


def complexity_curve(frames_list, heads, args):
    """Forward time under the radial list and under the all-ones list as the video grows (frames
    of the 720p geometry, s = 3600): the empirical form of the paper's O(n log n) claim (Fig. 2,
    Sec. 4.2 complexity analysis).  Prints one JSON line per length, then a summary line."""
    import dataclasses
    import numpy as np
    import torch
    from paper_2506_19852_amd import binding as rb
    from paper_2506_19852_amd import workloads as wl

    base = wl.WORKLOADS["cfg3_hunyuan720p"]
    width_num, width_den = (int(t) for t in args.width_scale.split("/"))
    rows = []
    for f in frames_list:
        w = dataclasses.replace(base, name=f"hunyuan720p_f{f}", frames=f, H=heads)
        x = {nm: wl.make_tensor(w, nm, "cuda:0") for nm in ("q", "k", "v")}
        out = torch.empty_like(x["q"])
        res = {}
        for kind in ("radial", "dense"):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            if kind == "radial":
                m = rb.radial_mask_build(w.frames, w.tokens_per_frame, w.block, 1, 0, width_num=width_num, width_den=width_den)
            else:
                m = rb.radial_mask_build_dense(w.N, w.block)
            torch.cuda.synchronize()
            build_ms = (time.perf_counter() - t0) * 1e3
            ptr, idx = rb.radial_mask_copy_to_host(m)
            flops = effective_flops(ptr, idx, w.N, w.block, w.D, w.B * w.H)
            rb.radial_attn_fwd(x["q"], x["k"], x["v"], out, None, m, w.scale)      # warm-up
            torch.cuda.synchronize()
            steps = args.steps if kind == "radial" else max(1, args.dense_steps)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(steps):
                rb.radial_attn_fwd(x["q"], x["k"], x["v"], out, None, m, w.scale)
            e1.record()
            torch.cuda.synchronize()
            res[kind] = {"pairs": int(ptr[-1]), "ms": e0.elapsed_time(e1) / steps, "flops": flops, "mask_build_ms": build_ms}
            m.free()
        r, d = res["radial"], res["dense"]
        row = {"frames": f, "N": w.N, "heads": heads, "listed_block_pairs": r["pairs"], "all_block_pairs": d["pairs"],
               "radial_ms": round(r["ms"], 3), "dense_ms": round(d["ms"], 3),
               "radial_tflops": round(r["flops"] / r["ms"] / 1e9, 1), "dense_tflops": round(d["flops"] / d["ms"] / 1e9, 1),
               "speedup_vs_dense": round(d["ms"] / r["ms"], 3), "block_ratio_dense_over_radial": round(d["flops"] / r["flops"], 3),
               "mask_build_ms": round(r["mask_build_ms"], 3)}
        rows.append(row)
        print(json.dumps(row), flush=True)
        del x, out
        torch.cuda.empty_cache()
    # growth exponents between the first and the last length: time ~ N^p
    a, b = rows[0], rows[-1]
    ln = np.log(b["N"] / a["N"])
    summary = {"curve": "forward time vs frames, s = 3600, block 128, D 128, width scale " + args.width_scale,
               "exponent_radial_time": round(float(np.log(b["radial_ms"] / a["radial_ms"]) / ln), 3),
               "exponent_dense_time": round(float(np.log(b["dense_ms"] / a["dense_ms"]) / ln), 3),
               "exponent_listed_pairs": round(float(np.log(b["listed_block_pairs"] / a["listed_block_pairs"]) / ln), 3),
               "pairs_per_n_log2f": [round(r["listed_block_pairs"] / (r["N"] / 128 * np.log2(r["frames"])), 2) for r in rows]}
    print(json.dumps(summary))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg3_hunyuan720p")
    ap.add_argument("--dense-steps", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--token-exact", action="store_true",
                    help="apply the token-level rule inside the listed blocks (same blocks computed; default: block-dense)")
    ap.add_argument("--width-scale", default="1/1", metavar="NUM/DEN",
                    help="sparsity knob: scales the diagonal width of frame pairs at distance >= 2 (default 1/1 = the printed mask)")
    ap.add_argument("--pattern", default="radial",
                    help="mask: radial (default), or a banded comparison mask: spatial:W (frames), temporal:H (positions), "
                         "sliding:W:H, harmonic")
    ap.add_argument("--fp8-scores", action="store_true",
                    help="forward with Q and K quantised to E4M3 per 128-token block (scores on the 8-bit matrix "
                         "instruction); a reduced-precision extra, never the headline number")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain device copy of q (known size) so a rocprofv3 --pmc run can scale FETCH_SIZE/WRITE_SIZE")
    ap.add_argument("--curve-frames", default=None, metavar="F1,F2,...",
                    help="instead of the benchmark line: forward time vs video length at the 720p geometry (s = 3600)")
    ap.add_argument("--curve-heads", type=int, default=2)
    ap.add_argument("--secondary", default="cfg2_wan480p,cfg4_hunyuan720p_4x,cfg5_wan480p_4x_bwd", metavar="W1,W2,...",
                    help="other workloads reported in the line's `secondary` array (kernel times only; 'none' to skip)")
    ap.add_argument("--secondary-launches", type=int, default=2)
    ap.add_argument("--mfma-probe-seconds", type=float, default=0.0,
                    help="after the benchmark, keep launching the MFMA-only probe for this long (for sampling board power and clock)")
    ap.add_argument("--cache-probe", action="store_true",
                    help="also run a streaming read of 2 GiB and 16 re-reads of a 64 MiB tensor (torch.neg), so that a "
                         "rocprofv3 --pmc TCC_EA0_RDREQ_sum TCC_EA0_RDREQ_LEVEL_sum run can compare the read latency seen "
                         "by the attention kernel's L2 misses with HBM reads and with reads the last-level cache serves")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    if args.curve_frames:
        complexity_curve([int(t) for t in args.curve_frames.split(",")], args.curve_heads, args)
        return

    import numpy as np
    import torch
    from paper_2506_19852_amd import binding as rb
    from paper_2506_19852_amd import workloads as wl

    w = wl.WORKLOADS[args.workload]
    width_num, width_den = (int(t) for t in args.width_scale.split("/"))
    dev = "cuda:0"
    torch.cuda.set_device(0)
    x = wl.make_inputs(w, dev)
    flags = rb.RADIAL_MASK_TRANSPOSE if w.backward else 0
    if args.token_exact:
        flags |= rb.RADIAL_MASK_TOKEN_EXACT
    out = torch.empty_like(x["q"])
    lse = torch.empty((w.B, w.H, w.N), dtype=torch.float32, device=dev)
    grads = ws = None
    if w.backward:
        grads = [torch.empty_like(x["q"]) for _ in range(3)]

    def build_mask():
        if args.pattern == "radial":
            return rb.radial_mask_build(w.frames, w.tokens_per_frame, w.block, 1, flags, width_num=width_num, width_den=width_den)
        from paper_2506_19852_amd import patterns
        kind, *par = args.pattern.split(":")
        par = [int(t) for t in par]
        table = {"spatial": patterns.spatial_head, "temporal": patterns.temporal_head,
                 "sliding": patterns.sliding_window, "harmonic": patterns.harmonic_decay}[kind](w.frames, w.tokens_per_frame, *par)
        return rb.radial_mask_build_banded(w.frames, w.tokens_per_frame, w.block, 1, table, flags)

    quant = None
    if args.fp8_scores:
        if w.backward or args.token_exact or w.block != 128 or w.D != 128:
            print("--fp8-scores: forward only, block 128, D 128, listed blocks dense", file=sys.stderr)
            sys.exit(2)
        nb = (w.N + w.block - 1) // w.block
        quant = {"qc": torch.empty(x["q"].shape, dtype=torch.uint8, device=dev), "kc": torch.empty(x["k"].shape, dtype=torch.uint8, device=dev),
                 "qs": torch.empty((w.B, w.H, nb), dtype=torch.float32, device=dev), "ks": torch.empty((w.B, w.H, nb), dtype=torch.float32, device=dev)}
        for _ in range(2):      # second pass timed
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            rb.radial_quantize_fp8(x["q"], w.block, quant["qc"], quant["qs"])
            rb.radial_quantize_fp8(x["k"], w.block, quant["kc"], quant["ks"])
            e1.record()
            torch.cuda.synchronize()
        quant["ms"] = e0.elapsed_time(e1)

    def forward(m, lse_out):
        if quant is not None:
            rb.radial_attn_fwd_fp8(quant["qc"], quant["qs"], quant["kc"], quant["ks"], x["v"], out, lse_out, m, w.scale)
        else:
            rb.radial_attn_fwd(x["q"], x["k"], x["v"], out, lse_out, m, w.scale)

    def step(keep=None):
        m = build_mask()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        forward(m, lse)
        e1.record()
        if w.backward:
            nonlocal ws
            if ws is None:
                ws = torch.empty(rb.radial_attn_bwd_workspace(w.B, w.H, w.N, w.D, m), dtype=torch.uint8, device=dev)
            rb.radial_attn_bwd(x["q"], x["k"], x["v"], out, x["do"], lse, *grads, m, w.scale, ws)
        if keep is not None:
            keep.append((m, e0, e1))
        else:
            torch.cuda.synchronize()
            m.free()

    if args.copy_probe:
        torch.neg(x["q"], out=out)     # one streaming kernel: reads and writes q.numel()*2 bytes
        torch.cuda.synchronize()
    if args.cache_probe:
        big = torch.zeros(1 << 30, dtype=torch.bfloat16, device=dev)      # 2 GiB: larger than every cache
        torch.neg(big, out=big)
        torch.cuda.synchronize()
        del big
        small = torch.zeros(32 << 20, dtype=torch.bfloat16, device=dev)   # 64 MiB: fits the last-level cache, not the L2s
        dst = torch.empty_like(small)
        for _ in range(16):
            torch.neg(small, out=dst)
        torch.cuda.synchronize()
        del small, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    keep = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(keep)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    launch_ms = [e0.elapsed_time(e1) for (_, e0, e1) in keep]
    kernel_ms = float(np.mean(launch_ms))
    row_ptr, col_idx = rb.radial_mask_copy_to_host(keep[0][0])
    for m, _, _ in keep:
        m.free()

    fwd_flops = effective_flops(row_ptr, col_idx, w.N, w.block, w.D, w.B * w.H)
    step_flops = fwd_flops * (3.5 if w.backward else 1.0)      # backward = 5 products vs 2
    ms_per_step = dt / args.steps * 1e3
    value = step_flops / (dt / args.steps) / 1e12

    # dense baseline: same kernel, all-ones list
    dense = rb.radial_mask_build_dense(w.N, w.block)
    dptr, didx = rb.radial_mask_copy_to_host(dense)
    dense_flops = effective_flops(dptr, didx, w.N, w.block, w.D, w.B * w.H)
    forward(dense, None)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.dense_steps):
        forward(dense, None)
    e1.record()
    torch.cuda.synchronize()
    dense_ms = e0.elapsed_time(e1) / args.dense_steps
    dense.free()

    # mask build alone (static mask: built once per video shape), host clock around a synchronised call
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    m = build_mask()
    torch.cuda.synchronize()
    mask_build_ms = (time.perf_counter() - t0) * 1e3

    # load balance: one traced launch, {begin, end, where} per workgroup
    balance = None
    if quant is None:
        trace = torch.zeros((rb.radial_attn_fwd_trace_records(w.B, w.H, m), 3), dtype=torch.int64, device=dev)
        rb.radial_attn_fwd_trace(x["q"], x["k"], x["v"], out, lse, m, w.scale, trace)
        torch.cuda.synchronize()
        balance = load_balance(trace.cpu().numpy())
        del trace
    keep_mask = m

    # the matrix pipes alone, at the clock the chip sustains: dependent MFMAs on registers
    probe_iters = 20000
    rb.radial_probe_mfma_bf16(probe_iters)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    probe_flops = rb.radial_probe_mfma_bf16(probe_iters)
    e1.record()
    torch.cuda.synchronize()
    probe_tflops = probe_flops / (e0.elapsed_time(e1) * 1e-3) / 1e12
    if args.mfma_probe_seconds > 0:   # keep the probe running so that an outside sampler can read clock and power
        t_end = time.perf_counter() + args.mfma_probe_seconds
        while time.perf_counter() < t_end:
            rb.radial_probe_mfma_bf16(probe_iters)
            torch.cuda.synchronize()

    achieved = fwd_flops / (kernel_ms * 1e-3) / 1e12
    traffic, traffic_source = None, None
    if width_num == width_den and not args.token_exact and args.pattern == "radial" and quant is None:
        traffic, traffic_source = traffic_from_profile(w.name, kernel_ms, float(x["q"].numel() * 2))
    result = {
        "metric": "effective TFLOP/s on computed blocks + speedup vs dense attn at same N, 1 GPU",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "fp8_e4m3 scores, bf16 PV" if quant is not None else "bf16", "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "H": w.H, "N": w.N, "D": w.D, "frames": w.frames,
                   "tokens_per_frame": w.tokens_per_frame, "block": w.block, "sink_frames": 1,
                   "listed_block_pairs": int(row_ptr[-1]), "pass": "fwd+bwd" if w.backward else "fwd",
                   "inside_listed_blocks": "token rule" if args.token_exact else "dense",
                   "width_scale": f"{width_num}/{width_den}", "pattern": args.pattern,
                   "block_sparsity": round(1.0 - float(row_ptr[-1]) / float((row_ptr.size - 1) ** 2), 4)},
        "fwd_kernel_ms": round(kernel_ms, 3),
        "fwd_kernel_ms_median": round(float(np.median(launch_ms)), 3), "fwd_kernel_ms_min": round(float(np.min(launch_ms)), 3),
        "mask_build_ms": round(mask_build_ms, 3),
        "mfma_probe_tflops": round(probe_tflops, 1),
        "load_balance": balance,
        "dense_fwd_kernel_ms": round(dense_ms, 3),
        "dense_tflops": round(dense_flops / (dense_ms * 1e-3) / 1e12, 2),
        "speedup_vs_dense": round(dense_ms / kernel_ms, 3),
        "block_ratio_dense_over_radial": round(dense_flops / fwd_flops, 3),
        "roofline": {"bound": "mfma", "achieved": round(achieved, 2), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(achieved / MFMA_BF16_PEAK_TFLOPS, 4), "frac_of_mfma_probe": round(achieved / probe_tflops, 4),
                     "traffic": traffic, "traffic_source": traffic_source,
                     "kernel": "radial_fwd_kernel", "flops_per_launch": fwd_flops},
    }
    if quant is not None:
        result["quantize_q_and_k_ms"] = round(quant["ms"], 3)
        result["roofline"]["kernel"] = "radial_fwd_fp8_kernel"
        result["roofline"]["traffic"] = None
        result["roofline"]["note"] = "half of the flops run on the 8-bit matrix instruction; peak and frac are still the bf16 figures"
    if not args.no_cpu_baseline:
        forward(keep_mask, None)                       # the result the oracle's sample is compared with
        torch.cuda.synchronize()
        result["cpu_baseline"] = cpu_baseline(w, x, row_ptr, col_idx, gpu_out=out)
    keep_mask.free()
    names = [] if args.secondary in ("", "none") or quant is not None or args.token_exact or args.pattern != "radial" \
        or width_num != width_den else [t for t in args.secondary.split(",") if t != w.name]
    if names:
        del x, out, lse, grads
        torch.cuda.empty_cache()
        result["secondary"] = []
        for nm in names:      # a failure here must not cost the headline line
            try:
                result["secondary"].append(secondary_config(nm, args, not args.no_cpu_baseline))
            except Exception as e:  # noqa: BLE001
                result["secondary"].append({"workload": nm, "error": f"{type(e).__name__}: {e}"})
                torch.cuda.empty_cache()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
