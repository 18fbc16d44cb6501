// Measurement aids (declared in include/radial_diag.h; no part of the method): the forward kernel
// built with per-workgroup trace records, and a kernel that only issues MFMAs.
#include "radial_attn_fwd_kernel.h"
#include "radial_diag.h"

namespace radial {
namespace {
// 4 waves per SIMD, each a chain of dependent 32x32x16 bf16 MFMAs on registers: the rate the
// matrix pipes sustain at the clock the chip holds, with no memory traffic at all.
__global__ void __launch_bounds__(1024) mfma_probe_kernel(int64_t iters, float* sink) {
  // operands: pseudo-random bf16 values in (-2, 2), four different A and B registers in turn, so
  // the multipliers see changing bits as they do on real data
  bf16x8 x[4], y[4];
  uint32_t r = threadIdx.x * 2654435761u + 12345u;
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      r = r * 1664525u + 1013904223u;
      x[j][i] = (__bf16)((float)(int)(r >> 16 & 0xFFFF) * (1.f / 16384.f) - 2.f);
      r = r * 1664525u + 1013904223u;
      y[j][i] = (__bf16)((float)(int)(r >> 16 & 0xFFFF) * (1.f / 16384.f) - 2.f);
    }
  f32x16 acc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;
  for (int64_t it = 0; it < iters; it += 4) {  // iters is a multiple of 4
#pragma unroll
    for (int rot = 0; rot < 4; ++rot)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x[j], y[(j + rot) & 3], acc[j], 0, 0, 0);
  }
  float t = 0.f;
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int e = 0; e < 16; ++e) t += acc[j][e];
  if (t == 0.12345f && sink != nullptr) sink[0] = t;  // keeps the chains alive; sink is null in every launch
}
constexpr int kProbeGrid = 256 * 8;  // 8 workgroups of 16 waves per compute unit
}  // namespace

int launch_mfma_probe(int64_t iters, hipStream_t stream, double* flops_out) {
  mfma_probe_kernel<<<dim3(kProbeGrid), dim3(1024), 0, stream>>>(iters, nullptr);
  RADIAL_HIP_TRY(hipGetLastError());
  if (flops_out) *flops_out = (double)kProbeGrid * 16.0 * (double)iters * 4.0 * (2.0 * 32 * 32 * 16);
  return RADIAL_OK;
}


}  // namespace radial

using namespace radial;

extern "C" int64_t radial_attn_fwd_trace_records(int32_t B, int32_t H, const radial_mask* mask) {
  if (!mask || B < 1 || H < 1) return 0;
  return 8LL * B * H * mask->max_slice;
}

extern "C" int radial_attn_fwd_trace(int32_t B, int32_t H, int32_t N, int32_t D, radial_tensor q, radial_tensor k,
                                     radial_tensor v, radial_tensor out, float* lse, const radial_mask* mask,
                                     float scale, void* hip_stream, uint64_t* trace, int64_t trace_records) {
  if (!trace) return fail(RADIAL_EINVAL, "trace is NULL");
  FwdArgs a;
  if (int rc = make_fwd_args(B, H, N, D, q, k, v, out, lse, mask, scale, &a)) return rc;
  if (trace_records < fwd_grid(a))
    return fail(RADIAL_ESHAPE, "trace holds %lld records, %lld needed", (long long)trace_records, (long long)fwd_grid(a));
  a.wg_trace = trace;
  return fwd::launch_any<true>(D, mask->block, a, (hipStream_t)hip_stream);
}

extern "C" int radial_probe_mfma_bf16(int64_t iterations, void* hip_stream, double* flops) {
  if (iterations < 4 || iterations > (1LL << 20) || (iterations & 3))
    return fail(RADIAL_EINVAL, "iterations must be a multiple of 4 in [4, 2^20]");
  return launch_mfma_probe(iterations, (hipStream_t)hip_stream, flops);
}
