/* libradial -- measurement aids.  No part of the method (arXiv 2506.19852 defines none of this):
 * the benchmark uses them for load-balance figures and for the matrix-pipe rate at the clock the
 * chip sustains.  Same conventions as radial.h. */
#ifndef RADIAL_DIAG_H_
#define RADIAL_DIAG_H_

#include "radial.h"

#ifdef __cplusplus
extern "C" {
#endif

/* radial_attn_fwd_trace is radial_attn_fwd plus one record per workgroup of the launch, for
 * load-balance figures: trace (device memory, trace_records x 3 uint64, zero-filled by the caller;
 * trace_records >= radial_attn_fwd_trace_records(B, H, mask), else RADIAL_ESHAPE) receives, for
 * every workgroup that had work, {begin, end, where}: begin and end in ticks of the device's
 * constant 100 MHz clock, where = (XCC_ID register << 32) | HW_ID register of the wave that wrote
 * it.  Workgroups without work leave their record untouched.  Same errors as radial_attn_fwd;
 * RADIAL_EINVAL if trace is NULL.  radial_attn_fwd_trace_records returns 0 on bad arguments. */
RADIAL_API int64_t radial_attn_fwd_trace_records(int32_t B, int32_t H, const radial_mask* mask);
RADIAL_API int radial_attn_fwd_trace(int32_t B, int32_t H, int32_t N, int32_t D, radial_tensor q, radial_tensor k,
                                     radial_tensor v, radial_tensor out, float* lse, const radial_mask* mask,
                                     float scale, void* hip_stream, uint64_t* trace, int64_t trace_records);

/* Launches, on hip_stream of the current device, a kernel that does nothing but dependent
 * 32x32x16 bf16 MFMAs on registers (16 waves per workgroup, 8 workgroups per compute unit,
 * 4 x iterations MFMAs per wave): timed by the caller, it gives the matrix-pipe rate at the clock
 * the chip sustains, the ceiling the attention kernels are compared with next to the published
 * peak.  *flops (host, may be NULL) receives the floating-point operations of the launch.
 * The operands are pseudo-random bf16 values that change from one MFMA to the next.
 * iterations: a multiple of 4 in [4, 2^20], else RADIAL_EINVAL.  Allocates nothing. */
RADIAL_API int radial_probe_mfma_bf16(int64_t iterations, void* hip_stream, double* flops);

#ifdef __cplusplus
}
#endif
#endif /* RADIAL_DIAG_H_ */
