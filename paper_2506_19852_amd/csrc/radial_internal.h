// Internal declarations shared by the libradial translation units (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "radial.h"

// Device-side description of a block list; owned by radial_mask.
struct radial_mask {
  int32_t n_tokens = 0;
  int32_t block = 0;
  int32_t n_blocks = 0;  // ceil(n_tokens / block): number of query blocks == number of key blocks
  int64_t nnz = 0;
  uint32_t flags = 0;
  int device = 0;
  // owners of the device storage; the pointers below are views into them
  int32_t* d_meta = nullptr;     // totals and launch partitions
  int32_t* d_ptrs = nullptr;     // row_ptr (+ col_ptr)
  int32_t* d_idx = nullptr;      // col_idx (+ row_idx)
  int32_t* d_row_ptr = nullptr;  // [n_blocks + 1]
  int32_t* d_col_idx = nullptr;  // [nnz]
  int32_t* d_col_ptr = nullptr;  // [n_blocks + 1]  (transpose; only with RADIAL_MASK_TRANSPOSE)
  int32_t* d_row_idx = nullptr;  // [nnz]
  // Launch partition: XCD x of the 8 works on query blocks [slice[x], slice[x+1]) of every
  // (batch, head), so that all XCDs are on the same head at the same time (its K/V then sit
  // in the shared last-level cache) and carry equal weight.  Same for key blocks (backward).
  int32_t* d_slice = nullptr;    // [9]
  int32_t* d_slice_t = nullptr;  // [9]
  int32_t max_slice = 0;         // longest slice, in blocks (host copy, sizes the grid)
  int32_t max_slice_t = 0;
  int32_t tokens_per_frame = 0;  // geometry of a radial mask (0 for dense / caller-supplied lists)
  int32_t sink_frames = 0;
  int32_t width_num = 1, width_den = 1;  // sparsity knob of a radial mask
  int32_t frames = 0;                    // video frames (tokens from frames*tokens_per_frame on are text tokens)
  int32_t* d_half_width = nullptr;       // [frames + 1] banded patterns only: half width per frame distance
};

namespace radial {

constexpr int kMaxDevices = 64;  // per-device tables of the library are this long

// Records a message for radial_last_error() and returns `code`.
int fail(int code, const char* fmt, ...);

#define RADIAL_HIP_TRY(expr)                                                              \
  do {                                                                                    \
    hipError_t e_ = (expr);                                                               \
    if (e_ != hipSuccess)                                                                 \
      return ::radial::fail(RADIAL_EHIP, "%s failed: %s", #expr, hipGetErrorString(e_));  \
  } while (0)

// Token-level rule of the radial mask, for kernels that apply it inside listed blocks.
struct TokenRule {
  int32_t exact;  // 0: listed blocks are dense
  int32_t s;      // tokens per frame
  int32_t sink;   // key frames below this are visible to everyone
  int32_t frames; // video frames; tokens of later "frames" are text tokens: they see and are seen by everyone
  // sparsity knob c = num/den for frame distances >= 2: the diagonal of band r is
  // floor(c*s / 2^r) = w0 >> r wide, with w0 = floor(s*num/den)
  int32_t w0;
  int32_t den;
  int64_t s_num;  // s * num
  const int32_t* half_width;  // banded patterns: device table by frame distance (null: radial rule)
};

inline TokenRule make_token_rule(const radial_mask* m) {
  TokenRule r;
  r.exact = (m->flags & RADIAL_MASK_TOKEN_EXACT) ? 1 : 0;
  r.s = m->tokens_per_frame;
  r.sink = m->sink_frames;
  r.frames = m->frames;
  r.s_num = (int64_t)m->tokens_per_frame * m->width_num;
  r.den = m->width_den;
  r.w0 = (int32_t)(r.s_num / m->width_den);
  r.half_width = m->d_half_width;
  return r;
}

struct TensorArg {
  const void* ptr;
  int64_t sb, sh, sn;  // element strides
};

struct FwdArgs {
  TensorArg q, k, v, o;
  float* lse;  // may be null
  const int32_t* row_ptr;
  const int32_t* col_idx;
  const int32_t* slice;  // [9] query-block partition over the XCDs
  int32_t max_slice;
  int32_t B, H, N, n_blocks;
  float scale;
  TokenRule rule;
  uint64_t* wg_trace;  // null, or [grid][3]: begin, end (100 MHz clock), where the workgroup ran
};

int launch_fwd(int D, int block, const FwdArgs& a, hipStream_t stream);
// Argument checks of a forward call (as radial_attn_fwd documents them); fills *a, wg_trace = null.
int make_fwd_args(int32_t B, int32_t H, int32_t N, int32_t D, radial_tensor q, radial_tensor k, radial_tensor v,
                  radial_tensor out, float* lse, const radial_mask* mask, float scale, FwdArgs* a);
// Workgroups one forward launch of this shape starts (the number of trace records).
int64_t fwd_grid(const FwdArgs& a);
// Launches a kernel that only issues dependent bf16 MFMAs from registers; *flops_out (host)
// receives the floating-point operations it performs.
int launch_mfma_probe(int64_t iters, hipStream_t stream, double* flops_out);

// 8-bit scores: Q and K as E4M3 codes ([B, H, N, D] bytes, contiguous) with one scale per
// (batch, head, block of tokens).
struct Fp8FwdArgs {
  const uint8_t* q8;
  const uint8_t* k8;
  const float* q_scale;  // [B, H, n_blocks]
  const float* k_scale;
  TensorArg v, o;
  float* lse;  // may be null
  const int32_t* row_ptr;
  const int32_t* col_idx;
  const int32_t* slice;
  int32_t max_slice;
  int32_t B, H, N, n_blocks;
  float scale;
};
int launch_fwd_fp8(const Fp8FwdArgs& a, hipStream_t stream);
int launch_quantize_fp8(int32_t B, int32_t H, int32_t N, int32_t D, const TensorArg& x, int32_t block, uint8_t* codes,
                        float* scales, hipStream_t stream);

struct BwdArgs {
  TensorArg q, k, v, o, dout, dq, dk, dv;
  const float* lse;
  float* delta;   // workspace: [B, H, N] rowsum(dO * O)
  const int32_t* row_ptr;
  const int32_t* col_idx;
  const int32_t* col_ptr;
  const int32_t* row_idx;
  const int32_t* slice;    // [9] query-block partition over the XCDs
  const int32_t* slice_t;  // [9] key-block partition over the XCDs
  int32_t max_slice, max_slice_t;
  int32_t B, H, N, n_blocks;
  float scale;
  TokenRule rule;
};

int launch_bwd(int D, int block, const BwdArgs& a, hipStream_t stream);

}  // namespace radial
