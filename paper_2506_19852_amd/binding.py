"""ctypes binding of libradial.so: same names as the C ABI in include/radial.h, argument
marshalling only.  Tensors are torch CUDA tensors (device memory + strides); every step of
the computation runs in the library's HIP kernels.  There is no fallback: a missing library
or a failing call raises."""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, byref, c_float, c_int32, c_int64, c_size_t, c_uint32, c_void_p

import numpy as np

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libradial.so")

RADIAL_MASK_TRANSPOSE = 1
RADIAL_MASK_TOKEN_EXACT = 2
STATUS = {0: "RADIAL_OK", -1: "RADIAL_EINVAL", -2: "RADIAL_ENOMEM", -3: "RADIAL_EHIP",
          -4: "RADIAL_EUNSUPPORTED", -5: "RADIAL_ESHAPE"}

EXPORTS = (
    "radial_last_error", "radial_mask_build", "radial_mask_build_banded", "radial_mask_build_dense", "radial_mask_from_csr",
    "radial_mask_info", "radial_mask_copy_to_host", "radial_mask_copy_transpose_to_host",
    "radial_mask_free", "radial_attn_fwd", "radial_attn_bwd_workspace", "radial_attn_bwd",
    "radial_attn_fwd_trace_records", "radial_attn_fwd_trace", "radial_probe_mfma_bf16",
    "radial_quantize_fp8", "radial_attn_fwd_fp8", "radial_attn_bwd_static",
)


class RadialError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"{STATUS.get(code, code)}: {message}")
        self.code = code


class radial_mask_params(ctypes.Structure):
    _fields_ = [("frames", c_int32), ("tokens_per_frame", c_int32), ("block", c_int32),
                ("sink_frames", c_int32), ("flags", c_uint32), ("width_num", c_int32), ("width_den", c_int32),
                ("extra_tokens", c_int32)]


class radial_tensor(ctypes.Structure):
    _fields_ = [("ptr", c_void_p), ("stride_b", c_int64), ("stride_h", c_int64), ("stride_n", c_int64)]


_lib = None


def lib_path() -> str:
    return _LIB_PATH


def load():
    """Loads libradial.so (built by paper_2506_19852_amd.build) and declares the prototypes."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: run `python -m paper_2506_19852_amd.build` (needs hipcc)")
    lib = ctypes.CDLL(_LIB_PATH)
    lib.radial_last_error.restype = ctypes.c_char_p
    lib.radial_last_error.argtypes = []
    lib.radial_mask_build.argtypes = [POINTER(radial_mask_params), c_void_p, POINTER(c_void_p)]
    lib.radial_mask_build_banded.argtypes = [c_int32, c_int32, c_int32, c_int32, POINTER(c_int32), c_uint32, c_void_p,
                                             POINTER(c_void_p)]
    lib.radial_mask_build_dense.argtypes = [c_int32, c_int32, c_uint32, c_void_p, POINTER(c_void_p)]
    lib.radial_mask_from_csr.argtypes = [c_int32, c_int32, c_uint32, c_void_p, c_void_p, c_void_p, POINTER(c_void_p)]
    lib.radial_mask_info.argtypes = [c_void_p, POINTER(c_int32), POINTER(c_int32), POINTER(c_int32),
                                     POINTER(c_int64), POINTER(c_uint32)]
    lib.radial_mask_copy_to_host.argtypes = [c_void_p, c_void_p, c_void_p]
    lib.radial_mask_copy_transpose_to_host.argtypes = [c_void_p, c_void_p, c_void_p]
    lib.radial_mask_free.argtypes = [c_void_p]
    lib.radial_mask_free.restype = None
    lib.radial_attn_fwd.argtypes = [c_int32, c_int32, c_int32, c_int32, radial_tensor, radial_tensor, radial_tensor,
                                    radial_tensor, c_void_p, c_void_p, c_float, c_void_p]
    lib.radial_attn_fwd_trace.argtypes = lib.radial_attn_fwd.argtypes + [c_void_p, ctypes.c_int64]
    lib.radial_attn_fwd_trace_records.argtypes = [c_int32, c_int32, c_void_p]
    lib.radial_attn_fwd_trace_records.restype = ctypes.c_int64
    lib.radial_probe_mfma_bf16.argtypes = [ctypes.c_int64, c_void_p, ctypes.POINTER(ctypes.c_double)]
    lib.radial_quantize_fp8.argtypes = [c_int32, c_int32, c_int32, c_int32, radial_tensor, c_int32, c_void_p, c_void_p, c_void_p]
    lib.radial_attn_fwd_fp8.argtypes = [c_int32, c_int32, c_int32, c_int32, c_int32, c_void_p, c_void_p, c_void_p, c_void_p,
                                        radial_tensor, radial_tensor, c_void_p, c_void_p, c_float, c_void_p]
    lib.radial_attn_bwd_workspace.argtypes = [c_int32, c_int32, c_int32, c_int32, c_void_p]
    lib.radial_attn_bwd_workspace.restype = c_size_t
    lib.radial_attn_bwd.argtypes = [c_int32, c_int32, c_int32, c_int32] + [radial_tensor] * 5 + [c_void_p] + \
        [radial_tensor] * 3 + [c_void_p, c_float, c_void_p, c_size_t, c_void_p]
    lib.radial_attn_bwd_static.argtypes = [c_int32, c_int32, c_int32, c_int32] + [radial_tensor] * 5 + [c_void_p] + \
        [radial_tensor] * 3 + [c_void_p, c_float, c_void_p]
    for name in EXPORTS:
        fn = getattr(lib, name)
        if name not in ("radial_last_error", "radial_mask_free", "radial_attn_bwd_workspace", "radial_attn_fwd_trace_records"):
            fn.restype = ctypes.c_int
    _lib = lib
    return lib


def radial_last_error() -> str:
    return load().radial_last_error().decode()


def _check(rc: int):
    if rc != 0:
        raise RadialError(rc, radial_last_error())


def _stream_ptr(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return c_void_p(int(getattr(stream, "cuda_stream", stream)))


class RadialMask:
    """Owner of a radial_mask* handle."""

    def __init__(self, handle):
        self._h = handle

    @property
    def handle(self):
        if not self._h:
            raise ValueError("mask was freed")
        return self._h

    def free(self):
        if self._h:
            load().radial_mask_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def radial_mask_build(frames: int, tokens_per_frame: int, block: int, sink_frames: int = 1, flags: int = 0,
                      stream=None, width_num: int = 1, width_den: int = 1, extra_tokens: int = 0) -> RadialMask:
    p = radial_mask_params(frames, tokens_per_frame, block, sink_frames, flags, width_num, width_den, extra_tokens)
    out = c_void_p()
    _check(load().radial_mask_build(byref(p), _stream_ptr(stream), byref(out)))
    return RadialMask(out)


def radial_mask_build_banded(frames: int, tokens_per_frame: int, block: int, sink_frames: int, half_width,
                             flags: int = 0, stream=None) -> RadialMask:
    hw = np.ascontiguousarray(half_width, dtype=np.int32)
    if hw.shape != (frames,):
        raise ValueError("half_width needs one entry per frame distance 0 .. frames-1")
    out = c_void_p()
    _check(load().radial_mask_build_banded(frames, tokens_per_frame, block, sink_frames,
                                           hw.ctypes.data_as(POINTER(c_int32)), flags, _stream_ptr(stream), byref(out)))
    return RadialMask(out)


def radial_mask_build_dense(n_tokens: int, block: int, flags: int = 0, stream=None) -> RadialMask:
    out = c_void_p()
    _check(load().radial_mask_build_dense(n_tokens, block, flags, _stream_ptr(stream), byref(out)))
    return RadialMask(out)


def radial_mask_from_csr(n_tokens: int, block: int, row_ptr, col_idx, flags: int = 0, stream=None) -> RadialMask:
    rp = np.ascontiguousarray(row_ptr, dtype=np.int32)
    ci = np.ascontiguousarray(col_idx, dtype=np.int32)
    out = c_void_p()
    _check(load().radial_mask_from_csr(n_tokens, block, flags, rp.ctypes.data, ci.ctypes.data if ci.size else None,
                                       _stream_ptr(stream), byref(out)))
    return RadialMask(out)


def radial_mask_info(mask: RadialMask) -> dict:
    n, blk, nb, nnz, fl = c_int32(), c_int32(), c_int32(), c_int64(), c_uint32()
    _check(load().radial_mask_info(mask.handle, byref(n), byref(blk), byref(nb), byref(nnz), byref(fl)))
    return {"n_tokens": n.value, "block": blk.value, "n_blocks": nb.value, "nnz": nnz.value, "flags": fl.value}


def radial_mask_copy_to_host(mask: RadialMask):
    info = radial_mask_info(mask)
    row_ptr = np.empty(info["n_blocks"] + 1, dtype=np.int32)
    col_idx = np.empty(info["nnz"], dtype=np.int32)
    _check(load().radial_mask_copy_to_host(mask.handle, row_ptr.ctypes.data, col_idx.ctypes.data if col_idx.size else None))
    return row_ptr, col_idx


def radial_mask_copy_transpose_to_host(mask: RadialMask):
    info = radial_mask_info(mask)
    col_ptr = np.empty(info["n_blocks"] + 1, dtype=np.int32)
    row_idx = np.empty(info["nnz"], dtype=np.int32)
    _check(load().radial_mask_copy_transpose_to_host(mask.handle, col_ptr.ctypes.data,
                                                     row_idx.ctypes.data if row_idx.size else None))
    return col_ptr, row_idx


def _tensor(t, name) -> radial_tensor:
    import torch
    if t.dtype != torch.bfloat16 or not t.is_cuda or t.dim() != 4 or t.stride(3) != 1:
        raise ValueError(f"{name} must be a CUDA bf16 tensor [B, H, N, D] with unit stride in D")
    return radial_tensor(t.data_ptr(), t.stride(0), t.stride(1), t.stride(2))


def radial_attn_fwd(q, k, v, out, lse, mask: RadialMask, scale: float, stream=None):
    """out[B,H,N,D] (bf16) and lse[B,H,N] (fp32, or None) <- block-sparse attention of q, k, v."""
    import torch
    B, H, N, D = q.shape
    for t, nm in ((k, "k"), (v, "v"), (out, "out")):
        if tuple(t.shape) != (B, H, N, D):
            raise ValueError(f"{nm} has shape {tuple(t.shape)}, expected {(B, H, N, D)}")
    lse_ptr = None
    if lse is not None:
        if lse.dtype != torch.float32 or not lse.is_cuda or not lse.is_contiguous() or tuple(lse.shape) != (B, H, N):
            raise ValueError("lse must be a contiguous CUDA float32 tensor [B, H, N]")
        lse_ptr = c_void_p(lse.data_ptr())
    _check(load().radial_attn_fwd(B, H, N, D, _tensor(q, "q"), _tensor(k, "k"), _tensor(v, "v"), _tensor(out, "out"),
                                  lse_ptr, mask.handle, c_float(scale), _stream_ptr(stream)))


def radial_attn_fwd_trace_records(B: int, H: int, mask: RadialMask) -> int:
    return int(load().radial_attn_fwd_trace_records(B, H, mask.handle))


def radial_attn_fwd_trace(q, k, v, out, lse, mask: RadialMask, scale: float, trace, stream=None):
    """radial_attn_fwd plus one {begin, end, where} record per workgroup in trace (zeroed CUDA int64 [records, 3])."""
    import torch
    B, H, N, D = q.shape
    if trace.dtype != torch.int64 or not trace.is_cuda or not trace.is_contiguous() or trace.dim() != 2 or trace.shape[1] != 3:
        raise ValueError("trace must be a contiguous CUDA int64 tensor [records, 3]")
    lse_ptr = c_void_p(lse.data_ptr()) if lse is not None else None
    _check(load().radial_attn_fwd_trace(B, H, N, D, _tensor(q, "q"), _tensor(k, "k"), _tensor(v, "v"), _tensor(out, "out"),
                                        lse_ptr, mask.handle, c_float(scale), _stream_ptr(stream),
                                        c_void_p(trace.data_ptr()), trace.shape[0]))


def radial_probe_mfma_bf16(iterations: int, stream=None) -> float:
    """Launches the MFMA-only probe kernel; returns the floating-point operations it performs."""
    flops = ctypes.c_double(0.0)
    _check(load().radial_probe_mfma_bf16(iterations, _stream_ptr(stream), ctypes.byref(flops)))
    return flops.value


def radial_quantize_fp8(x, block: int, codes, scales, stream=None):
    """codes (uint8 [B,H,N,D]) and scales (float32 [B,H,ceil(N/block)]) <- per-block E4M3 quantisation of x (bf16)."""
    import torch
    B, H, N, D = x.shape
    nb = (N + block - 1) // block
    if codes.dtype != torch.uint8 or not codes.is_cuda or not codes.is_contiguous() or tuple(codes.shape) != (B, H, N, D):
        raise ValueError("codes must be a contiguous CUDA uint8 tensor [B, H, N, D]")
    if scales.dtype != torch.float32 or not scales.is_cuda or not scales.is_contiguous() or tuple(scales.shape) != (B, H, nb):
        raise ValueError("scales must be a contiguous CUDA float32 tensor [B, H, ceil(N/block)]")
    _check(load().radial_quantize_fp8(B, H, N, D, _tensor(x, "x"), block, c_void_p(codes.data_ptr()),
                                      c_void_p(scales.data_ptr()), _stream_ptr(stream)))


def radial_attn_fwd_fp8(q_codes, q_scales, k_codes, k_scales, v, out, lse, mask: RadialMask, scale: float, stream=None,
                        code_block: int = 128):
    """radial_attn_fwd with the scores computed from E4M3 codes of q and k made by radial_quantize_fp8
    with block = code_block."""
    import torch
    B, H, N, D = v.shape
    nb = (N + code_block - 1) // code_block
    for t, nm in ((q_codes, "q_codes"), (k_codes, "k_codes")):
        if t.dtype != torch.uint8 or not t.is_cuda or not t.is_contiguous() or tuple(t.shape) != (B, H, N, D):
            raise ValueError(f"{nm} must be a contiguous CUDA uint8 tensor [B, H, N, D]")
    for t, nm in ((q_scales, "q_scales"), (k_scales, "k_scales")):
        if t.dtype != torch.float32 or not t.is_cuda or not t.is_contiguous() or tuple(t.shape) != (B, H, nb):
            raise ValueError(f"{nm} must be a contiguous CUDA float32 tensor [B, H, ceil(N/code_block)]")
    if tuple(out.shape) != (B, H, N, D):
        raise ValueError("out has the wrong shape")
    lse_ptr = None
    if lse is not None:
        if lse.dtype != torch.float32 or not lse.is_cuda or not lse.is_contiguous() or tuple(lse.shape) != (B, H, N):
            raise ValueError("lse must be a contiguous CUDA float32 tensor [B, H, N]")
        lse_ptr = c_void_p(lse.data_ptr())
    _check(load().radial_attn_fwd_fp8(B, H, N, D, code_block, c_void_p(q_codes.data_ptr()), c_void_p(q_scales.data_ptr()),
                                      c_void_p(k_codes.data_ptr()), c_void_p(k_scales.data_ptr()), _tensor(v, "v"),
                                      _tensor(out, "out"), lse_ptr, mask.handle, c_float(scale), _stream_ptr(stream)))


def radial_attn_bwd_workspace(B: int, H: int, N: int, D: int, mask: RadialMask) -> int:
    return int(load().radial_attn_bwd_workspace(B, H, N, D, mask.handle))


def radial_attn_bwd(q, k, v, out, dout, lse, dq, dk, dv, mask: RadialMask, scale: float, workspace, stream=None):
    """dq, dk, dv <- gradient of the block-sparse attention; workspace: CUDA uint8 tensor."""
    B, H, N, D = q.shape
    ts = [_tensor(t, nm) for t, nm in ((q, "q"), (k, "k"), (v, "v"), (out, "out"), (dout, "dout"))]
    gs = [_tensor(t, nm) for t, nm in ((dq, "dq"), (dk, "dk"), (dv, "dv"))]
    _check(load().radial_attn_bwd(B, H, N, D, *ts, c_void_p(lse.data_ptr()), *gs, mask.handle, c_float(scale),
                                  c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size(),
                                  _stream_ptr(stream)))


def radial_attn_bwd_static(q, k, v, out, dout, lse, dq, dk, dv, mask: RadialMask, scale: float, stream=None):
    """radial_attn_bwd without a workspace: the library's own device array holds the row sums."""
    B, H, N, D = q.shape
    ts = [_tensor(t, nm) for t, nm in ((q, "q"), (k, "k"), (v, "v"), (out, "out"), (dout, "dout"))]
    gs = [_tensor(t, nm) for t, nm in ((dq, "dq"), (dk, "dk"), (dv, "dv"))]
    _check(load().radial_attn_bwd_static(B, H, N, D, *ts, c_void_p(lse.data_ptr()), *gs, mask.handle, c_float(scale),
                                         _stream_ptr(stream)))
