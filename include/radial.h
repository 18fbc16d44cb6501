/* libradial -- Radial Attention hot path for AMD MI355X (gfx950), C ABI.
 *
 * Implements, on one GPU, the two operations of "Radial Attention" (arXiv 2506.19852):
 *
 *   1. the static spatiotemporal mask of Sec. 4.2 ("Formal definition", with the attention
 *      sink of App. A.1) reduced to square blocks (Sec. 4.2, "Hardware-friendly block
 *      sparsity"), emitted as a compressed per-query-block list of key-block indices;
 *   2. SparseAttention(Q,K,V) = softmax((Q K^T + M)/sqrt(d)) V  (Sec. 3, Eq. 2) for the block
 *      mask M of (1), forward and backward, on bf16 [B,H,N,D] tensors.  With the all-ones
 *      list it is the dense attention of Eq. 1.
 *
 * Conventions
 *   - Every function returns RADIAL_OK (0) or a negative radial_status; nothing throws or
 *     aborts.  radial_last_error() returns a thread-local, NUL-terminated description of the
 *     last failure on the calling thread (valid until that thread's next failing call).
 *   - "device pointer" = memory of the current HIP device; "host pointer" = ordinary memory.
 *   - hip_stream is a hipStream_t passed as void* (NULL = the default stream).  Attention
 *     calls are asynchronous on that stream; mask construction returns after the lists are
 *     complete on the device.
 *   - Between calls the library keeps only what a radial_mask owns, a per-device note that a
 *     kernel attribute has been set, and the device array of radial_attn_bwd_static.
 */
#ifndef RADIAL_H_
#define RADIAL_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#if defined(__GNUC__)
#define RADIAL_API __attribute__((visibility("default")))
#else
#define RADIAL_API
#endif

typedef enum {
  RADIAL_OK = 0,
  RADIAL_EINVAL = -1,       /* NULL where a pointer is required, bad parameter value, unsorted list   */
  RADIAL_ENOMEM = -2,       /* host or device allocation failed                                      */
  RADIAL_EHIP = -3,         /* a HIP runtime call failed; radial_last_error() carries its message    */
  RADIAL_EUNSUPPORTED = -4, /* block or head dimension outside {64, 128}; more blocks or listed pairs than
                               the lists can index; token rule with frames shorter than 64 tokens   */
  RADIAL_ESHAPE = -5        /* tensor shape / stride / workspace does not match the mask or the call */
} radial_status;

RADIAL_API const char* radial_last_error(void);

/* ---- mask ------------------------------------------------------------------------------- */

/* Parameters of the radial mask.  Tokens are ordered frame-major: token (i, k) = frame i,
 * spatial position k, flattened index i*tokens_per_frame + k (Sec. 4.2, flattening rule).
 * Query token (i,k) may attend key token (j,l) iff, with d = |i-j| and b = 2^floor(log2 max(d,1)),
 *      j < sink_frames                                   (attention sink, App. A.1), or
 *      b <= s and (|k-l| + 1) * b <= s                   (first case of the formal definition), or
 *      d mod ceil(b/s) == 0 and k == l                   (second case).
 * Sparsity knob (the paper adjusts the mask's sparsity to a compute budget, Sec. 5.1 and
 * App. D, without defining how; this is the reading taken here): for frame pairs with d >= 2
 * the spatial extent is scaled by c = width_num / width_den, i.e. `s` in the two cases above
 * is replaced by c*s:  b*width_den <= s*width_num and (|k-l|+1)*b*width_den <= s*width_num,
 * or  d mod ceil(b*width_den / (s*width_num)) == 0 and k == l.  c = 1 is the printed mask.
 * Text tokens (the video models of Sec. 5.1 append prompt tokens to the video sequence; the
 * paper does not say how the mask treats them; reading taken here): `extra_tokens` tokens that
 * follow the video tokens attend to every token and are attended by every token.
 * Blocks of `block` consecutive flattened tokens tile [0, N) from 0 (the last one may be
 * ragged, and a block may straddle frames).  A (query block, key block) pair is listed iff
 * at least one of its token pairs may attend; a listed pair is computed densely. */
typedef struct {
  int32_t frames;           /* f >= 1                                                    */
  int32_t tokens_per_frame; /* s >= 1;  N = f*s must be < 2^31 - block                   */
  int32_t block;            /* 64 or 128                                                 */
  int32_t sink_frames;      /* >= 0; the paper uses 1; 0 disables the sink               */
  uint32_t flags;           /* RADIAL_MASK_* bits, others must be 0                      */
  int32_t width_num;        /* sparsity knob c = width_num / width_den: both in [1, 32767] */
  int32_t width_den;        /*   and tokens_per_frame * width_num < 2^31; 1, 1 = the paper */
  int32_t extra_tokens;     /* >= 0 text tokens after the f*s video tokens: N = f*s + extra */
} radial_mask_params;

#define RADIAL_MASK_TRANSPOSE 1u /* also build the per-key-block list of query blocks (needed by bwd) */
/* radial_mask_build only: attention calls with this mask apply the token-level rule above
 * inside the listed blocks as well, i.e. they evaluate Eq. 2 under the token mask of Sec. 4.2
 * itself instead of its block cover.  Needs tokens_per_frame >= 64 (EUNSUPPORTED otherwise). */
#define RADIAL_MASK_TOKEN_EXACT 2u

/* Opaque.  Owns device copies of row_ptr[nqb+1], col_idx[nnz] (and the transposed lists when
 * requested) plus a launch order for the attention kernels.  Immutable after construction;
 * may be shared by any number of attention calls and streams on the device it was built on.
 * The mask does not depend on B, H or D. */
typedef struct radial_mask radial_mask;

/* Builds the radial block lists with integer kernels on the GPU.  *out receives a new mask
 * that the caller releases with radial_mask_free.  Errors: EINVAL (NULL, f<1, s<1, sink<0,
 * extra_tokens<0, knob out of range, unknown flag, N too large), EUNSUPPORTED (block, more
 * than 491 520 key blocks, more than 2^31-1 listed pairs, token rule with s < 64), ENOMEM, EHIP. */
RADIAL_API int radial_mask_build(const radial_mask_params* params, void* hip_stream, radial_mask** out);

/* A banded static mask: query token (i,k) may attend key token (j,l) iff j < sink_frames or
 * |k - l| <= half_width[|i - j|]  (an entry of -1 hides the whole frame pair).  This one rule
 * covers the other static video masks the paper compares with (Sec. 3 and Sec. 5.1: the
 * "spatial" and "temporal" head masks, sliding windows; App., comparison with other
 * O(n log n) patterns: widths inversely proportional to the frame distance) and, while every
 * width is at least one, the radial mask itself.  The paper defines none of them formally;
 * the caller chooses the widths.
 *   half_width : host, int32 [frames], read during the call only;
 *   flags      : RADIAL_MASK_TRANSPOSE, RADIAL_MASK_TOKEN_EXACT (needs tokens_per_frame >= 64);
 *   block lists as for radial_mask_build ("any" cover, ascending, ragged last block).
 * Errors: EINVAL (NULL, f<1, s<1, sink<0, unknown flag, N too large), EUNSUPPORTED (block,
 * token rule with short frames), ENOMEM, EHIP. */
RADIAL_API int radial_mask_build_banded(int32_t frames, int32_t tokens_per_frame, int32_t block, int32_t sink_frames,
                                        const int32_t* half_width, uint32_t flags, void* hip_stream,
                                        radial_mask** out);

/* The all-ones list over ceil(n_tokens/block)^2 block pairs: dense attention, Eq. 1.
 * `flags` as in radial_mask_params. */
RADIAL_API int radial_mask_build_dense(int32_t n_tokens, int32_t block, uint32_t flags, void* hip_stream,
                            radial_mask** out);

/* A caller-supplied list.  row_ptr [nqb+1] and col_idx [row_ptr[nqb]] are HOST pointers,
 * copied.  Each row must be strictly ascending with entries in [0, nqb); row_ptr[0] == 0 and
 * non-decreasing (else EINVAL).  Rows may be empty. */
RADIAL_API int radial_mask_from_csr(int32_t n_tokens, int32_t block, uint32_t flags, const int32_t* row_ptr,
                         const int32_t* col_idx, void* hip_stream, radial_mask** out);

/* Any out-pointer may be NULL.  n_blocks = ceil(n_tokens/block); nnz = listed block pairs. */
RADIAL_API int radial_mask_info(const radial_mask* mask, int32_t* n_tokens, int32_t* block, int32_t* n_blocks,
                     int64_t* nnz, uint32_t* flags);

/* Copies the lists to HOST arrays row_ptr [n_blocks+1], col_idx [nnz] (either may be NULL).
 * Entries of a row ascend. */
RADIAL_API int radial_mask_copy_to_host(const radial_mask* mask, int32_t* row_ptr, int32_t* col_idx);

/* Same for the transposed lists (col_ptr [n_blocks+1], row_idx [nnz]): for each key block the
 * ascending query blocks that list it.  ESHAPE if the mask was built without
 * RADIAL_MASK_TRANSPOSE. */
RADIAL_API int radial_mask_copy_transpose_to_host(const radial_mask* mask, int32_t* col_ptr, int32_t* row_idx);

/* NULL-safe.  Must not be called while an attention call that uses the mask is in flight. */
RADIAL_API void radial_mask_free(radial_mask* mask);

/* ---- attention ---------------------------------------------------------------------------- */

/* A bf16 tensor of logical shape [B, H, N, D] on the device: element (b,h,n,d) lives at
 * ptr + 2*(b*stride_b + h*stride_h + n*stride_n + d) bytes; strides are in elements, the
 * innermost (D) stride is 1, stride_n >= D, ptr and every row start 16-byte aligned
 * (all strides multiples of 8).  The caller owns the memory. */
typedef struct {
  void* ptr;
  int64_t stride_b, stride_h, stride_n;
} radial_tensor;

/* Forward, Eq. 2:  out = softmax(scale * Q K^T restricted to the listed blocks) V.
 *   q, k, v : inputs;  out : output (may not alias the inputs);
 *   lse     : device float [B, H, N] contiguous, receives log(sum_k exp(scale * q.k)) over the
 *             visible keys of each row (needed by radial_attn_bwd), or NULL;
 *   scale   : the 1/sqrt(d) of Eq. 2 (any positive finite value is accepted).
 * Inside a listed block pair every key with index < N is visible; with a mask built under
 * RADIAL_MASK_TOKEN_EXACT only the pairs the token rule allows are.  A query row with no
 * visible key gets out = 0 and lse = -inf.  Products run on bf16 MFMA with fp32 accumulation;
 * the softmax is fp32; P is rounded to bf16 before P.V; out is rounded to nearest-even bf16.
 * Allocates nothing (the call can be captured into a HIP graph).
 * Errors: EINVAL (NULL, scale), EUNSUPPORTED (D not 64/128), ESHAPE (N != mask n_tokens,
 * misaligned pointer/stride, B*H*n_blocks >= 2^31), EHIP. */
RADIAL_API int radial_attn_fwd(int32_t B, int32_t H, int32_t N, int32_t D, radial_tensor q, radial_tensor k,
                    radial_tensor v, radial_tensor out, float* lse, const radial_mask* mask,
                    float scale, void* hip_stream);

/* Bytes of device workspace radial_attn_bwd needs for this problem (0 on invalid arguments). */
RADIAL_API size_t radial_attn_bwd_workspace(int32_t B, int32_t H, int32_t N, int32_t D, const radial_mask* mask);

/* Backward of Eq. 2 for the scalar loss whose gradient w.r.t. `out` is `dout`:
 *   P = exp(scale*Q K^T - lse) on listed blocks,  dV = P^T dO,  dP = dO V^T,
 *   delta = rowsum(dO * O),  dS = P * (dP - delta),  dQ = scale * dS K,  dK = scale * dS^T Q.
 *   out, lse : as produced by radial_attn_fwd with the same q, k, v, mask, scale;
 *   dq, dk, dv : outputs, bf16, fully overwritten;
 *   workspace : device memory of at least radial_attn_bwd_workspace(...) bytes, 256-byte
 *               aligned, contents ignored on entry and undefined on return.
 * The mask must carry RADIAL_MASK_TRANSPOSE (ESHAPE otherwise).  Allocates nothing. */
RADIAL_API int radial_attn_bwd(int32_t B, int32_t H, int32_t N, int32_t D, radial_tensor q, radial_tensor k,
                    radial_tensor v, radial_tensor out, radial_tensor dout, const float* lse,
                    radial_tensor dq, radial_tensor dk, radial_tensor dv, const radial_mask* mask,
                    float scale, void* workspace, size_t workspace_bytes, void* hip_stream);

/* radial_attn_bwd for callers that cannot allocate device memory or carry a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * results and errors as radial_attn_bwd without `workspace`: the per-row sums live in a device
 * array of RADIAL_BWD_STATIC_MAX_BYTES that is part of the library's code object (each GPU the
 * library runs on holds it until the process ends).  RADIAL_ESHAPE if
 * radial_attn_bwd_workspace(B, H, N, D, mask) exceeds RADIAL_BWD_STATIC_MAX_BYTES, i.e. if
 * B*H*N > 6 291 456.  Calls no hipMalloc/hipFree; the first call on a device looks up the
 * array's address.  All calls on one GPU share the array: calls whose kernels may overlap there
 * (different streams, or several host threads) race; order them on one stream. */
#define RADIAL_BWD_STATIC_MAX_BYTES (24u << 20)
RADIAL_API int radial_attn_bwd_static(int32_t B, int32_t H, int32_t N, int32_t D, radial_tensor q, radial_tensor k,
                    radial_tensor v, radial_tensor out, radial_tensor dout, const float* lse,
                    radial_tensor dq, radial_tensor dk, radial_tensor dv, const radial_mask* mask,
                    float scale, void* hip_stream);

/* ---- 8-bit scores (optional) -------------------------------------------------------------------
 *
 * The paper defines no quantisation (Sec. 2 and Sec. 6 call the method orthogonal to quantised
 * attention kernels); this scheme is the library's own.  Q and K are cut into blocks of `block`
 * consecutive tokens of one (batch, head); a block is stored as E4M3 codes (OCP 8-bit floating
 * point: 4 exponent bits, bias 7, 3 mantissa bits, largest value 448, round to nearest even) of
 * x / scale with scale = amax / 448 (1 for an all-zero block), all in float32.
 *
 * radial_quantize_fp8: x is a [B, H, N, D] bf16 tensor (strided like q), D a multiple of 8;
 * codes (device, B*H*N*D bytes, contiguous [B, H, N, D], 16-byte aligned) and scales (device,
 * B*H*ceil(N/block) floats, [B, H, block index]) are written.  Errors: RADIAL_EINVAL (NULL,
 * sizes < 1), RADIAL_EUNSUPPORTED (D), RADIAL_ESHAPE (strides, alignment), RADIAL_EHIP.
 *
 * radial_attn_fwd_fp8 is radial_attn_fwd (Eq. 2 on the listed blocks, listed blocks dense) with
 * the scores computed from such codes: S = (q codes . k codes) * q scale * k scale on the 8-bit
 * matrix instruction; the softmax, P (bf16) and the product with V (bf16) are unchanged.
 * code_block is the `block` the codes and scales were made with by radial_quantize_fp8; it must
 * equal the mask's block (RADIAL_ESHAPE otherwise: the scales would be read per wrong block).  Only D = 128 with block 128, and
 * not for masks with RADIAL_MASK_TOKEN_EXACT (RADIAL_EUNSUPPORTED otherwise); other errors as
 * radial_attn_fwd.  Allocates nothing. */
RADIAL_API int radial_quantize_fp8(int32_t B, int32_t H, int32_t N, int32_t D, radial_tensor x, int32_t block,
                                   uint8_t* codes, float* scales, void* hip_stream);
RADIAL_API int radial_attn_fwd_fp8(int32_t B, int32_t H, int32_t N, int32_t D, int32_t code_block, const uint8_t* q_codes,
                                   const float* q_scales, const uint8_t* k_codes, const float* k_scales,
                                   radial_tensor v, radial_tensor out, float* lse, const radial_mask* mask,
                                   float scale, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* RADIAL_H_ */
