"""Seeded synthetic workloads (inputs only -- none of the method's arithmetic lives here).

The five configurations mirror the video-DiT attention shapes the paper evaluates on
(Wan2.1-14B and HunyuanVideo token grids, Sec. 5.1); real activations are replaced by
iid N(0,1) tensors with 3-D rotary position embedding applied to q and k.  Values come from
a counter-based generator (a 64-bit mix of seed, tensor id and element index followed by
Box-Muller), evaluated with torch integer/float ops on whichever device is asked for; the
tensors are rounded to bf16 once and those exact bytes go to both the GPU library and the
CPU oracle.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import torch

SEED0 = 0x5241444941


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    H: int
    D: int
    frames: int
    grid_h: int
    grid_w: int
    block: int
    rope: bool
    backward: bool
    seed: int

    @property
    def tokens_per_frame(self) -> int:
        return self.grid_h * self.grid_w

    @property
    def N(self) -> int:
        return self.frames * self.tokens_per_frame

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.D)


WORKLOADS = {
    # tiny: 8 frames x 256 tokens, block 64, no RoPE
    "cfg1_tiny": Workload("cfg1_tiny", 1, 2, 64, 8, 16, 16, 64, False, False, SEED0 + 1),
    # Wan-14B-shaped 480p layer: 21 latent frames x (30 x 52)
    "cfg2_wan480p": Workload("cfg2_wan480p", 1, 40, 128, 21, 30, 52, 128, True, False, SEED0 + 2),
    # HunyuanVideo-shaped 720p default length: 33 latent frames x (45 x 80)
    "cfg3_hunyuan720p": Workload("cfg3_hunyuan720p", 1, 24, 128, 33, 45, 80, 128, True, False, SEED0 + 3),
    # HunyuanVideo-shaped 4x longer video: 129 latent frames
    "cfg4_hunyuan720p_4x": Workload("cfg4_hunyuan720p_4x", 1, 24, 128, 129, 45, 80, 128, True, False, SEED0 + 4),
    # Wan-shaped 4x longer 480p, forward + backward
    "cfg5_wan480p_4x_bwd": Workload("cfg5_wan480p_4x_bwd", 1, 40, 128, 81, 30, 52, 128, True, True, SEED0 + 5),
}

_M1 = 0xBF58476D1CE4E5B9 - (1 << 64)     # as signed int64 (torch has no uint64 arithmetic)
_M2 = 0x94D049BB133111EB - (1 << 64)


def _signed64(x: int) -> int:
    x &= (1 << 64) - 1
    return x - (1 << 64) if x >> 63 else x


def _lsr(x: torch.Tensor, k: int) -> torch.Tensor:
    """Logical right shift of int64 bit patterns."""
    return (x >> k) & ((1 << (64 - k)) - 1)


def _mix64(x: torch.Tensor) -> torch.Tensor:
    x = (x ^ _lsr(x, 30)) * _M1
    x = (x ^ _lsr(x, 27)) * _M2
    return x ^ _lsr(x, 31)


def normal_from_counter(seed: int, tensor_id: int, start: int, count: int, device) -> torch.Tensor:
    """count iid N(0,1) float32 values for element indices start .. start+count-1."""
    idx = torch.arange(start, start + count, dtype=torch.int64, device=device)
    key = _signed64((seed * 0x100 + tensor_id) * 0x9E3779B97F4A7C15)
    h1 = _mix64(idx * 2 + key)
    h2 = _mix64(idx * 2 + 1 + key)
    u1 = (_lsr(h1, 11).to(torch.float64) + 1.0) * (1.0 / 9007199254740992.0)      # (0, 1]
    u2 = _lsr(h2, 11).to(torch.float64) * (1.0 / 9007199254740992.0)              # [0, 1)
    r = torch.sqrt(-2.0 * torch.log(u1))
    return (r * torch.cos(2.0 * math.pi * u2)).to(torch.float32)


def rope_3d(x: torch.Tensor, frames: int, grid_h: int, grid_w: int, dims=(16, 56, 56), theta: float = 1e4) -> torch.Tensor:
    """Rotary embedding over (t, h, w) for x [N, D] float32, tokens ordered t-major then h then w.

    The head dimension is split into three axis groups; inside a group of size a, the pair
    (2m, 2m+1) is rotated by angle pos * theta^(-2m/a), pos being the integer grid index."""
    n, d = x.shape
    assert sum(dims) == d and n == frames * grid_h * grid_w
    tok = torch.arange(n, device=x.device)
    pos = (tok // (grid_h * grid_w), (tok // grid_w) % grid_h, tok % grid_w)
    out = torch.empty_like(x)
    base = 0
    for axis, a in enumerate(dims):
        m = torch.arange(a // 2, device=x.device, dtype=torch.float64)
        freq = theta ** (-2.0 * m / a)
        ang = pos[axis].to(torch.float64)[:, None] * freq[None, :]
        c, s = torch.cos(ang).to(torch.float32), torch.sin(ang).to(torch.float32)
        xe, xo = x[:, base:base + a:2], x[:, base + 1:base + a:2]
        out[:, base:base + a:2] = xe * c - xo * s
        out[:, base + 1:base + a:2] = xe * s + xo * c
        base += a
    return out


TENSOR_IDS = {"q": 1, "k": 2, "v": 3, "do": 4}


def make_tensor(w: Workload, which: str, device, heads=None) -> torch.Tensor:
    """bf16 tensor [B, H, N, D] (or only the listed heads: [B, len(heads), N, D]) of workload w."""
    heads = list(range(w.H)) if heads is None else list(heads)
    out = torch.empty((w.B, len(heads), w.N, w.D), dtype=torch.bfloat16, device=device)
    per_head = w.N * w.D
    for b in range(w.B):
        for hi, h in enumerate(heads):
            start = (b * w.H + h) * per_head
            x = normal_from_counter(w.seed, TENSOR_IDS[which], start, per_head, device).view(w.N, w.D)
            if w.rope and which in ("q", "k"):
                x = rope_3d(x, w.frames, w.grid_h, w.grid_w)
            out[b, hi] = x.to(torch.bfloat16)
    return out


def make_inputs(w: Workload, device, heads=None):
    names = ["q", "k", "v"] + (["do"] if w.backward else [])
    return {nm: make_tensor(w, nm, device, heads) for nm in names}
