// C-ABI entry points of the attention calls: argument checks, then the kernel launchers.
#include <math.h>

#include <mutex>

#include "radial_internal.h"

using namespace radial;

namespace {

int check_tensor(const char* name, const radial_tensor& t, int32_t D) {
  if (!t.ptr) return fail(RADIAL_EINVAL, "%s.ptr is NULL", name);
  if (((uintptr_t)t.ptr & 15u) != 0) return fail(RADIAL_ESHAPE, "%s.ptr is not 16-byte aligned", name);
  if (t.stride_n < D || (t.stride_n & 7) || (t.stride_h & 7) || (t.stride_b & 7) || t.stride_h < 0 || t.stride_b < 0)
    return fail(RADIAL_ESHAPE, "%s strides must be non-negative multiples of 8 elements with stride_n >= D", name);
  if (t.stride_n >= (1 << 22)) return fail(RADIAL_ESHAPE, "%s.stride_n must be below 2^22 elements", name);
  return RADIAL_OK;
}

int check_call(int32_t B, int32_t H, int32_t N, int32_t D, const radial_mask* mask, float scale) {
  if (!mask) return fail(RADIAL_EINVAL, "mask is NULL");
  if (B < 1 || H < 1 || N < 1) return fail(RADIAL_EINVAL, "B, H, N must be >= 1");
  if (D != 64 && D != 128) return fail(RADIAL_EUNSUPPORTED, "head dimension must be 64 or 128 (got %d)", D);
  if (N != mask->n_tokens) return fail(RADIAL_ESHAPE, "N = %d but the mask was built for %d tokens", N, mask->n_tokens);
  if (!(scale > 0.f) || !isfinite(scale)) return fail(RADIAL_EINVAL, "scale must be positive and finite");
  if ((int64_t)B * H * mask->n_blocks >= 0x7fffffffLL - 8) return fail(RADIAL_ESHAPE, "B*H*n_blocks does not fit one launch");
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev != mask->device)
    return fail(RADIAL_ESHAPE, "mask lives on device %d, current device is %d", mask->device, dev);
  return RADIAL_OK;
}

TensorArg arg(const radial_tensor& t) { return TensorArg{t.ptr, t.stride_b, t.stride_h, t.stride_n}; }

}  // namespace

// Argument checks of a forward call; fills *a (without trace records).
int radial::make_fwd_args(int32_t B, int32_t H, int32_t N, int32_t D, radial_tensor q, radial_tensor k, radial_tensor v,
                          radial_tensor out, float* lse, const radial_mask* mask, float scale, FwdArgs* a) {
  if (int rc = check_call(B, H, N, D, mask, scale)) return rc;
  if (int rc = check_tensor("q", q, D)) return rc;
  if (int rc = check_tensor("k", k, D)) return rc;
  if (int rc = check_tensor("v", v, D)) return rc;
  if (int rc = check_tensor("out", out, D)) return rc;
  a->q = arg(q); a->k = arg(k); a->v = arg(v); a->o = arg(out);
  a->lse = lse;
  a->row_ptr = mask->d_row_ptr;
  a->col_idx = mask->d_col_idx;
  a->slice = mask->d_slice;
  a->max_slice = mask->max_slice;
  a->B = B; a->H = H; a->N = N; a->n_blocks = mask->n_blocks;
  a->scale = scale;
  a->rule = make_token_rule(mask);
  a->wg_trace = nullptr;
  return RADIAL_OK;
}

extern "C" int radial_attn_fwd(int32_t B, int32_t H, int32_t N, int32_t D, radial_tensor q, radial_tensor k,
                               radial_tensor v, radial_tensor out, float* lse, const radial_mask* mask, float scale,
                               void* hip_stream) {
  FwdArgs a;
  if (int rc = make_fwd_args(B, H, N, D, q, k, v, out, lse, mask, scale, &a)) return rc;
  return launch_fwd(D, mask->block, a, (hipStream_t)hip_stream);
}

// Workspace layout: delta [B*H*N] fp32.
static size_t delta_bytes(int32_t B, int32_t H, int32_t N) {
  const size_t raw = (size_t)B * H * N * sizeof(float);
  return (raw + 255) & ~(size_t)255;
}

extern "C" size_t radial_attn_bwd_workspace(int32_t B, int32_t H, int32_t N, int32_t D, const radial_mask* mask) {
  if (!mask || B < 1 || H < 1 || N < 1 || (D != 64 && D != 128) || N != mask->n_tokens) return 0;
  return delta_bytes(B, H, N);
}

// Checks and launch shared by the two backward entry points; `delta` is device memory for
// B*H*N floats.
static int bwd_call(int32_t B, int32_t H, int32_t N, int32_t D, radial_tensor q, radial_tensor k, radial_tensor v,
                    radial_tensor out, radial_tensor dout, const float* lse, radial_tensor dq, radial_tensor dk,
                    radial_tensor dv, const radial_mask* mask, float scale, float* delta, void* hip_stream) {
  BwdArgs a;
  a.q = arg(q); a.k = arg(k); a.v = arg(v); a.o = arg(out); a.dout = arg(dout);
  a.dq = arg(dq); a.dk = arg(dk); a.dv = arg(dv);
  a.lse = lse;
  a.delta = delta;
  a.row_ptr = mask->d_row_ptr; a.col_idx = mask->d_col_idx;
  a.col_ptr = mask->d_col_ptr; a.row_idx = mask->d_row_idx;
  a.slice = mask->d_slice; a.max_slice = mask->max_slice;
  a.slice_t = mask->d_slice_t; a.max_slice_t = mask->max_slice_t;
  a.B = B; a.H = H; a.N = N; a.n_blocks = mask->n_blocks;
  a.scale = scale;
  a.rule = make_token_rule(mask);
  return launch_bwd(D, mask->block, a, (hipStream_t)hip_stream);
}

static int check_bwd(int32_t B, int32_t H, int32_t N, int32_t D, radial_tensor q, radial_tensor k, radial_tensor v,
                     radial_tensor out, radial_tensor dout, const float* lse, radial_tensor dq, radial_tensor dk,
                     radial_tensor dv, const radial_mask* mask, float scale) {
  if (int rc = check_call(B, H, N, D, mask, scale)) return rc;
  if (!(mask->flags & RADIAL_MASK_TRANSPOSE)) return fail(RADIAL_ESHAPE, "mask was built without RADIAL_MASK_TRANSPOSE");
  if (!lse) return fail(RADIAL_EINVAL, "lse is NULL");
  const radial_tensor* ts[] = {&q, &k, &v, &out, &dout, &dq, &dk, &dv};
  const char* names[] = {"q", "k", "v", "out", "dout", "dq", "dk", "dv"};
  for (int i = 0; i < 8; ++i)
    if (int rc = check_tensor(names[i], *ts[i], D)) return rc;
  return RADIAL_OK;
}

extern "C" int radial_attn_bwd(int32_t B, int32_t H, int32_t N, int32_t D, radial_tensor q, radial_tensor k,
                               radial_tensor v, radial_tensor out, radial_tensor dout, const float* lse,
                               radial_tensor dq, radial_tensor dk, radial_tensor dv, const radial_mask* mask,
                               float scale, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (int rc = check_bwd(B, H, N, D, q, k, v, out, dout, lse, dq, dk, dv, mask, scale)) return rc;
  const size_t need = radial_attn_bwd_workspace(B, H, N, D, mask);
  if (!workspace || ((uintptr_t)workspace & 255u)) return fail(RADIAL_ESHAPE, "workspace must be a 256-byte aligned device pointer");
  if (workspace_bytes < need) return fail(RADIAL_ESHAPE, "workspace holds %zu bytes, %zu needed", workspace_bytes, need);
  return bwd_call(B, H, N, D, q, k, v, out, dout, lse, dq, dk, dv, mask, scale, (float*)workspace, hip_stream);
}

// ---- backward without a workspace argument --------------------------------------------------
// The per-row sums `delta` live in a device array that is part of the library's code object:
// every GPU the library runs on holds its own copy, at its own address, until the process ends.
// The array's name below is only the host-side handle of that symbol; kernels get the device
// address that hipGetSymbolAddress returns for the current device.
static __device__ __align__(256) unsigned char scratch[RADIAL_BWD_STATIC_MAX_BYTES];

namespace {
std::mutex scratch_mutex;
void* scratch_ptr[kMaxDevices];  // device address of `scratch`, per device; null until first use there

// Device address of `scratch` on the current device (looked up once per device).
int scratch_on_current_device(void** out) {
  int dev = -1;
  RADIAL_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(RADIAL_EUNSUPPORTED, "device index %d is beyond the %d the library tracks", dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(scratch_mutex);
  if (!scratch_ptr[dev]) {
    void* p = nullptr;
    RADIAL_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p || ((uintptr_t)p & 255u)) return fail(RADIAL_EHIP, "the library's device scratch array has no usable address");
    scratch_ptr[dev] = p;
  }
  *out = scratch_ptr[dev];
  return RADIAL_OK;
}
}  // namespace

extern "C" int radial_attn_bwd_static(int32_t B, int32_t H, int32_t N, int32_t D, radial_tensor q, radial_tensor k,
                                      radial_tensor v, radial_tensor out, radial_tensor dout, const float* lse,
                                      radial_tensor dq, radial_tensor dk, radial_tensor dv, const radial_mask* mask,
                                      float scale, void* hip_stream) {
  if (int rc = check_bwd(B, H, N, D, q, k, v, out, dout, lse, dq, dk, dv, mask, scale)) return rc;
  const size_t need = radial_attn_bwd_workspace(B, H, N, D, mask);
  if (need == 0 || need > (size_t)RADIAL_BWD_STATIC_MAX_BYTES)
    return fail(RADIAL_ESHAPE, "B*H*N = %lld rows need %zu bytes of scratch; radial_attn_bwd_static holds %zu (use radial_attn_bwd)",
                (long long)B * H * N, need, (size_t)RADIAL_BWD_STATIC_MAX_BYTES);
  void* delta = nullptr;
  if (int rc = scratch_on_current_device(&delta)) return rc;
  // Every row of delta that the kernels read is written first by the prepare kernel of this same
  // call, so nothing has to be cleared; what an earlier call left behind is never read.
  return bwd_call(B, H, N, D, q, k, v, out, dout, lse, dq, dk, dv, mask, scale, (float*)delta, hip_stream);
}

extern "C" int radial_quantize_fp8(int32_t B, int32_t H, int32_t N, int32_t D, radial_tensor x, int32_t block,
                                   uint8_t* codes, float* scales, void* hip_stream) {
  if (B < 1 || H < 1 || N < 1) return fail(RADIAL_EINVAL, "B, H, N must be >= 1");
  if (D < 8 || (D & 7)) return fail(RADIAL_EUNSUPPORTED, "head dimension must be a positive multiple of 8 (got %d)", D);
  if (block < 1) return fail(RADIAL_EINVAL, "block must be >= 1");
  if (int rc = check_tensor("x", x, D)) return rc;
  if (!codes || !scales) return fail(RADIAL_EINVAL, "codes or scales is NULL");
  if ((uintptr_t)codes & 15u) return fail(RADIAL_ESHAPE, "codes is not 16-byte aligned");
  return launch_quantize_fp8(B, H, N, D, arg(x), block, codes, scales, (hipStream_t)hip_stream);
}

extern "C" int radial_attn_fwd_fp8(int32_t B, int32_t H, int32_t N, int32_t D, int32_t code_block, const uint8_t* q_codes, const float* q_scales,
                                   const uint8_t* k_codes, const float* k_scales, radial_tensor v, radial_tensor out,
                                   float* lse, const radial_mask* mask, float scale, void* hip_stream) {
  if (int rc = check_call(B, H, N, D, mask, scale)) return rc;
  if (D != 128 || mask->block != 128) return fail(RADIAL_EUNSUPPORTED, "8-bit scores need head dimension 128 and block 128");
  if (code_block != mask->block)
    return fail(RADIAL_ESHAPE, "codes were quantised per %d tokens, the mask's block is %d", code_block, mask->block);
  if (mask->flags & RADIAL_MASK_TOKEN_EXACT) return fail(RADIAL_EUNSUPPORTED, "8-bit scores do not apply the token rule inside blocks");
  if (!q_codes || !k_codes || !q_scales || !k_scales) return fail(RADIAL_EINVAL, "codes or scales is NULL");
  if (((uintptr_t)q_codes | (uintptr_t)k_codes) & 15u) return fail(RADIAL_ESHAPE, "codes are not 16-byte aligned");
  if (int rc = check_tensor("v", v, D)) return rc;
  if (int rc = check_tensor("out", out, D)) return rc;
  Fp8FwdArgs a;
  a.q8 = q_codes; a.k8 = k_codes; a.q_scale = q_scales; a.k_scale = k_scales;
  a.v = arg(v); a.o = arg(out);
  a.lse = lse;
  a.row_ptr = mask->d_row_ptr;
  a.col_idx = mask->d_col_idx;
  a.slice = mask->d_slice;
  a.max_slice = mask->max_slice;
  a.B = B; a.H = H; a.N = N; a.n_blocks = mask->n_blocks;
  a.scale = scale;
  return launch_fwd_fp8(a, (hipStream_t)hip_stream);
}
