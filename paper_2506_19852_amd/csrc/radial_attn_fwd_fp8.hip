// 8-bit scores for gfx950: per-block E4M3 quantisation of Q and K, and the block-sparse forward
// (Eq. 2 of the paper on the listed key blocks) with S = Q K^T on the fp8 matrix instruction.
// The paper leaves quantisation to other work (it calls the method orthogonal to quantised
// attention); the scheme is this library's own: a block of `block` consecutive tokens of one
// (batch, head) is stored as E4M3 codes of x / scale, scale = amax / 448.
//
// The forward kernel is the bf16 one with a different first product:
//     S^T[key, q] = scale_k scale_q  K8[key, :] . Q8[q, :]   on v_mfma_f32_32x32x64_f8f6f4
// (A = K8 tile from LDS, B = Q8^T in registers, 64 bytes of d per instruction: lane l supplies
// bytes 32*(l/32) .. +31 of the 64-byte slice for row/column l%32, the same bytes on both
// sides).  Its accumulator layout equals the bf16 instruction's, so the softmax, the second
// product (P in bf16, V in bf16) and the epilogue are unchanged.  The two scales are positive and
// constant over a stage, so they are folded into the exponent's multiplier and applied to the row
// maximum once per stage instead of to every score.
#include "radial_internal.h"
#include "radial_tile.h"

namespace radial {
namespace {

constexpr int kStageKeys = 64;
constexpr int D = 128, BLK = 128;
constexpr int kWaves = BLK / 32, kThreads = 64 * kWaves;
constexpr int kSubs = BLK / kStageKeys;
constexpr int kK8Bytes = kStageKeys * D;        // one K stage tile, 1 byte per element
constexpr int kVBytes = kStageKeys * D * 2;     // one V stage tile, bf16
constexpr int kBufBytes = kK8Bytes + kVBytes;
constexpr int kKLoads = kK8Bytes / 1024 / kWaves;   // 1 KiB copies per wave: 2
constexpr int kVLoads = kVBytes / 1024 / kWaves;    // 4
constexpr int kKeyTiles = kStageKeys / 32;
constexpr int kDTiles = D / 32;
using VT = SwzTile<D>;

typedef int i32x8 __attribute__((ext_vector_type(8)));

// K8 tile: rows of 128 bytes = 8 pieces of 16 bytes, two rows per 256-byte line; pieces are
// XOR-swizzled inside their line so that the 128-bit reads of one piece column over 16
// consecutive rows touch 16 different 16-byte bank groups.
__device__ __forceinline__ int k8_piece(int r, int p) {
  const int lin = r * 8 + p;
  const int line = lin >> 4, slot = lin & 15;
  return (line << 8) + ((slot ^ (line & 7)) << 4);
}
// (row, piece) of the source that belongs at linear LDS piece index `lin`
__device__ __forceinline__ void k8_source_of(int lin, int& r, int& p) {
  const int line = lin >> 4, slot = lin & 15;
  const int src = (line << 4) + (slot ^ (line & 7));
  r = src >> 3;
  p = src & 7;
}

// One workgroup per (batch*head, block of tokens): amax, scale, codes.
__global__ void __launch_bounds__(256) quantize_fp8_kernel(TensorArg x, uint8_t* codes, float* scales, int32_t H, int32_t N,
                                                           int32_t Dh, int32_t block, int32_t nb) {
  __shared__ float part[4];
  const int32_t bh = blockIdx.x / nb, blk = blockIdx.x % nb;
  const int32_t b = bh / H, h = bh % H;
  const __bf16* src = (const __bf16*)x.ptr + (int64_t)b * x.sb + (int64_t)h * x.sh;
  const int32_t row0 = blk * block;
  const int32_t rows = N - row0 < block ? N - row0 : block;
  const int32_t per_row = Dh / 8;                 // 16-byte pieces per row
  const int32_t pieces = rows * per_row;
  float amax = 0.f;
  for (int32_t i = threadIdx.x; i < pieces; i += 256) {
    const int32_t r = i / per_row, p = i % per_row;
    const bf16x8 v = *(const bf16x8*)(src + (int64_t)(row0 + r) * x.sn + 8 * p);
#pragma unroll
    for (int e = 0; e < 8; ++e) amax = fmaxf(amax, fabsf((float)v[e]));
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off));
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = amax;
  __syncthreads();
  amax = fmaxf(fmaxf(part[0], part[1]), fmaxf(part[2], part[3]));
  const float scale = amax > 0.f ? amax / 448.f : 1.f;
  if (threadIdx.x == 0) scales[(int64_t)bh * nb + blk] = scale;
  uint8_t* dst = codes + ((int64_t)bh * N + row0) * Dh;
  for (int32_t i = threadIdx.x; i < pieces; i += 256) {
    const int32_t r = i / per_row, p = i % per_row;
    const bf16x8 v = *(const bf16x8*)(src + (int64_t)(row0 + r) * x.sn + 8 * p);
    float y[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) y[e] = fminf(fmaxf((float)v[e] / scale, -448.f), 448.f);
    int lo = 0, hi = 0;  // v_cvt_pk_fp8_f32 rounds to nearest even; beyond the clamp it would give NaN
    lo = __builtin_amdgcn_cvt_pk_fp8_f32(y[0], y[1], lo, false);
    lo = __builtin_amdgcn_cvt_pk_fp8_f32(y[2], y[3], lo, true);
    hi = __builtin_amdgcn_cvt_pk_fp8_f32(y[4], y[5], hi, false);
    hi = __builtin_amdgcn_cvt_pk_fp8_f32(y[6], y[7], hi, true);
    *(u32x2*)(dst + (int64_t)r * Dh + 8 * p) = u32x2{(uint32_t)lo, (uint32_t)hi};
  }
}

__global__ void __launch_bounds__(kThreads, 3) radial_fwd_fp8_kernel(const Fp8FwdArgs a) {
  // [stage buffer][K8 tile, V tile]
  __shared__ __attribute__((aligned(1024))) char lds[2 * kBufBytes];
  const uint32_t lds_base = lds_address(lds);

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lq = lane & 31;
  const int g = lane >> 5;

  // Workgroup -> (batch*head, query block): as in the bf16 kernel (8 slices of equal list weight,
  // XCD x takes slice (x + head) mod 8, the XCDs move from head to head together).
  const int32_t xcd = blockIdx.x & 7;
  const int64_t idx = blockIdx.x >> 3;
  const int32_t bh = (int32_t)(idx / a.max_slice);
  const int32_t pos = (int32_t)(idx % a.max_slice);
  const int32_t sl = (xcd + bh) & 7;
  const int32_t s0 = a.slice[sl];
  if (pos >= a.slice[sl + 1] - s0) return;
  const int32_t qb = s0 + pos;
  const int32_t b = bh / a.H, h = bh % a.H;

  const uint8_t* qp = a.q8 + (int64_t)bh * a.N * D;
  const uint8_t* kp = a.k8 + (int64_t)bh * a.N * D;
  const __bf16* vp = (const __bf16*)a.v.ptr + (int64_t)b * a.v.sb + (int64_t)h * a.v.sh;
  __bf16* op = (__bf16*)a.o.ptr + (int64_t)b * a.o.sb + (int64_t)h * a.o.sh;
  const float* k_scale = a.k_scale + (int64_t)bh * a.n_blocks;
  const float q_scale = a.q_scale[(int64_t)bh * a.n_blocks + qb];

  const int32_t list_lo = __builtin_amdgcn_readfirstlane(a.row_ptr[qb]);
  const int32_t n_list = __builtin_amdgcn_readfirstlane(a.row_ptr[qb + 1]) - list_lo;
  const int32_t n_stage = n_list * kSubs;
  const int32_t q_row = qb * BLK + wave * 32 + lq;
  const bool q_ok = q_row < a.N;

  // Q8^T fragments: for the 64-byte slice t of d this lane holds bytes 64t + 32g .. +31 of its row.
  i32x8 qf[2];
  {
    const uint8_t* src = qp + (int64_t)(q_ok ? q_row : a.N - 1) * D + 32 * g;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      u32x4 r0 = *(const u32x4*)(src + 64 * t), r1 = *(const u32x4*)(src + 64 * t + 16);
      if (!q_ok) r0 = r1 = u32x4{0u, 0u, 0u, 0u};
      qf[t] = i32x8{(int)r0[0], (int)r0[1], (int)r0[2], (int)r0[3], (int)r1[0], (int)r1[1], (int)r1[2], (int)r1[3]};
    }
  }

  // List entries and the scales of their key blocks, 64 at a time in one register per lane.
  const int32_t* cols = a.col_idx + list_lo;
  int32_t cvec = lane < n_list ? cols[lane] : 0;
  int32_t nvec = 64 + lane < n_list ? cols[64 + lane] : 0;
  float csc = lane < n_list ? k_scale[cvec] : 1.f;
  float nsc = 64 + lane < n_list ? k_scale[nvec] : 1.f;

  // Which piece of a stage tile each of this lane's copies fetches, as a byte offset from the
  // first row of the tile.
  int32_t krow[kKLoads], vrow_[kVLoads], vcol[kVLoads];
  uint32_t koff[kKLoads], voff[kVLoads];
#pragma unroll
  for (int i = 0; i < kKLoads; ++i) {
    int r, p;
    k8_source_of((wave * kKLoads + i) * 64 + lane, r, p);
    krow[i] = r;
    koff[i] = (uint32_t)(r * D + p * 16);
  }
#pragma unroll
  for (int i = 0; i < kVLoads; ++i) {
    int r, c;
    VT::source_of((wave * kVLoads + i) * 64 + lane, r, c);
    vrow_[i] = r;
    vcol[i] = c;
    voff[i] = (uint32_t)(r * (int32_t)a.v.sn + c) * 2u;
  }
  // All copies of the stage that starts at key `key0` into stage buffer `buf`, at once.  Rows
  // past N-1 are clamped to N-1; their scores are masked before the softmax.
  auto issue_stage = [&](int32_t key0, int buf) {
    const uint32_t kdst = lds_base + buf * kBufBytes + wave * kKLoads * 1024;
    const uint32_t vdst = lds_base + buf * kBufBytes + kK8Bytes + wave * kVLoads * 1024;
    if (key0 + kStageKeys <= a.N) {
      const uint8_t* kbase = kp + (int64_t)key0 * D;
      const __bf16* vbase = vp + (int64_t)key0 * a.v.sn;
#pragma unroll
      for (int i = 0; i < kKLoads; ++i) copy16_to_lds_sv(kbase, koff[i], kdst + i * 1024);
#pragma unroll
      for (int i = 0; i < kVLoads; ++i) copy16_to_lds_sv(vbase, voff[i], vdst + i * 1024);
    } else {
      const int32_t last = a.N - 1 - key0;  // >= 0: a listed block starts below N
#pragma unroll
      for (int i = 0; i < kKLoads; ++i) {
        const int32_t r = krow[i] < last ? krow[i] : last;
        copy16_to_lds(kp + ((int64_t)key0 + r) * D + (koff[i] - (uint32_t)krow[i] * D), kdst + i * 1024);
      }
#pragma unroll
      for (int i = 0; i < kVLoads; ++i) {
        const int32_t r = vrow_[i] < last ? vrow_[i] : last;
        copy16_to_lds(vp + ((int64_t)key0 + r) * a.v.sn + vcol[i], vdst + i * 1024);
      }
    }
  };

  f32x16 o[kDTiles];
#pragma unroll
  for (int i = 0; i < kDTiles; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) o[i][e] = 0.f;
  float m_run = -INFINITY;  // running row maximum of the raw scores q.k (scales applied, softmax scale not)
  float l_run = 0.f;
  const float c = a.scale * 1.4426950408889634f;

  int32_t key0 = 0;
  float f_stage = 1.f;  // scale_q * scale_k of the stage about to be computed
  if (n_stage > 0) {
    key0 = __builtin_amdgcn_readlane(cvec, 0) * BLK;
    f_stage = q_scale * __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, csc), 0));
    issue_stage(key0, 0);
  }

  for (int32_t u = 0; u < n_stage; ++u) {
    const int buf = u & 1;
    int32_t key0_next = 0;
    float f_next = 1.f;
    const bool has_next = u + 1 < n_stage;
    if (has_next) {
      const int32_t e1 = (u + 1) / kSubs;
      if ((u + 1) % kSubs == 0 && (e1 & 63) == 0) {  // entering the next chunk of the list
        cvec = nvec;
        csc = nsc;
        nvec = e1 + 64 + lane < n_list ? cols[e1 + 64 + lane] : 0;
        nsc = e1 + 64 + lane < n_list ? k_scale[nvec] : 1.f;
      }
      key0_next = __builtin_amdgcn_readlane(cvec, e1 & 63) * BLK + ((u + 1) % kSubs) * kStageKeys;
      f_next = q_scale * __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, csc), e1 & 63));
    }

    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this wave's copies of stage u have landed
    __syncthreads();                                  // ... and everyone's; stage u-1 is fully consumed

    // Copies of stage u+1: K pieces between the MFMAs of the first product, V pieces between
    // those of the second; a ragged next stage is issued in one go.
    const bool spread = has_next && key0_next + kStageKeys <= a.N;
    if (has_next && !spread) issue_stage(key0_next, buf ^ 1);
    const uint32_t on = __builtin_amdgcn_readfirstlane(spread ? ~0u : 0u);
    const uint64_t lanes = ((uint64_t)on << 32) | on;
    const int32_t key_src = spread ? key0_next : key0;  // any valid rows when switched off
    const uint8_t* kbase_next = kp + (int64_t)key_src * D;
    const __bf16* vbase_next = vp + (int64_t)key_src * a.v.sn;
    const uint32_t kdst_next = lds_base + (buf ^ 1) * kBufBytes + wave * kKLoads * 1024;
    const uint32_t vdst_next = lds_base + (buf ^ 1) * kBufBytes + kK8Bytes + wave * kVLoads * 1024;
    const char* lds_k = lds + buf * kBufBytes;
    const char* lds_v = lds_k + kK8Bytes;

    // ---- S^T = K8 Q8^T (unscaled code products) ---------------------------------------------
    f32x16 s[kKeyTiles];
#pragma unroll
    for (int kt = 0; kt < kKeyTiles; ++kt) {
#pragma unroll
      for (int e = 0; e < 16; ++e) s[kt][e] = 0.f;
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const u32x4 k0 = *lds_cast<const u32x4>(lds_k + k8_piece(kt * 32 + lq, 4 * t + 2 * g));
        const u32x4 k1 = *lds_cast<const u32x4>(lds_k + k8_piece(kt * 32 + lq, 4 * t + 2 * g + 1));
        const i32x8 kf = {(int)k0[0], (int)k0[1], (int)k0[2], (int)k0[3], (int)k1[0], (int)k1[1], (int)k1[2], (int)k1[3]};
        // formats 0 / 0 = E4M3 for both operands; scale exponents 127 = 2^0
        s[kt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(kf, qf[t], s[kt], 0, 0, 0, 0x7F7F7F7F, 0, 0x7F7F7F7F);
        if (t == 1) copy16_to_lds_sv_masked(kbase_next, koff[kt], kdst_next + kt * 1024, lanes);
      }
    }

    // ---- online softmax ------------------------------------------------------------------
    // s[kt][e] belongs to key key0 + 32kt + 8(e/4) + 4g + e%4 and query q_row; keys >= N do not exist.
    if (key0 + kStageKeys > a.N) {
      const uint32_t hidden = ~lane_element_bits(stage_prefix(a.N - key0), g);
#pragma unroll
      for (int kt = 0; kt < kKeyTiles; ++kt)
#pragma unroll
        for (int e = 0; e < 16; ++e)
          if ((hidden >> (16 * kt + e)) & 1u) s[kt][e] = -INFINITY;
    }
    float mx = s[0][0];
#pragma unroll
    for (int kt = 0; kt < kKeyTiles; ++kt)
#pragma unroll
      for (int e = 0; e < 16; ++e) mx = fmaxf(mx, s[kt][e]);
    mx = max_with_other_half(mx) * f_stage;  // the scales are positive: they commute with the maximum
    const float m_new = fmaxf(m_run, mx);
    if (__builtin_amdgcn_ballot_w64(m_new > m_run) != 0) {
      const float alpha = m_new > m_run ? __builtin_amdgcn_exp2f((m_run - m_new) * c) : 1.f;
      l_run *= alpha;
#pragma unroll
      for (int i = 0; i < kDTiles; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[i][e] *= alpha;
      m_run = m_new;
    }
    const float mc = m_run == -INFINITY ? 0.f : m_run * c;
    const float cs = c * f_stage;
    float psum = 0.f;
    uint32_t pk[kKeyTiles][8];
#pragma unroll
    for (int kt = 0; kt < kKeyTiles; ++kt)
#pragma unroll
      for (int e = 0; e < 16; e += 2) {
        const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kt][e], cs, -mc));
        const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kt][e + 1], cs, -mc));
        psum += p0 + p1;
        pk[kt][e >> 1] = pack_bf16(p0, p1);
      }
    l_run += psum;

    // ---- O^T += V^T P^T --------------------------------------------------------------------
#pragma unroll
    for (int kt = 0; kt < kKeyTiles; ++kt)
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const bf16x8 pf = as_bf16x8(pk[kt][4 * t], pk[kt][4 * t + 1], pk[kt][4 * t + 2], pk[kt][4 * t + 3]);
#pragma unroll
        for (int dt = 0; dt < kDTiles; ++dt) {
          const int i16 = lane & 15;
          const int vrow = kt * 32 + 16 * t + 4 * g + (i16 >> 2);
          const int dcol = 32 * dt + 16 * ((lane >> 4) & 1) + 4 * (i16 & 3);
          const u32x2 a0 = lds_read_tr(lds_v + VT::elem(vrow, dcol)), a1 = lds_read_tr(lds_v + VT::elem(vrow + 8, dcol));
          const u32x4 vraw = {a0[0], a0[1], a1[0], a1[1]};
          o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vraw), pf, o[dt], 0, 0, 0);
          if (dt == 0) {
            const int j = kt * 2 + t;  // one V piece per four MFMAs
            copy16_to_lds_sv_masked(vbase_next, voff[j], vdst_next + j * 1024, lanes);
          }
        }
      }
    key0 = key0_next;
    f_stage = f_next;
  }

  // ---- epilogue: O / l, LSE ----------------------------------------------------------------
  const float l_tot = l_run + __shfl_xor(l_run, 32);
  const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
  if (q_ok) {
    __bf16* dst = op + (int64_t)q_row * a.o.sn;
#pragma unroll
    for (int dt = 0; dt < kDTiles; ++dt)
#pragma unroll
      for (int e4 = 0; e4 < 4; ++e4) {
        u32x2 w;
        w[0] = pack_bf16(o[dt][4 * e4] * inv, o[dt][4 * e4 + 1] * inv);
        w[1] = pack_bf16(o[dt][4 * e4 + 2] * inv, o[dt][4 * e4 + 3] * inv);
        *(u32x2*)(dst + 32 * dt + 8 * e4 + 4 * g) = w;
      }
    if (a.lse && g == 0) a.lse[(int64_t)bh * a.N + q_row] = l_tot > 0.f ? m_run * a.scale + __logf(l_tot) : -INFINITY;
  }
}

}  // namespace

int launch_quantize_fp8(int32_t B, int32_t H, int32_t N, int32_t Dh, const TensorArg& x, int32_t block, uint8_t* codes,
                        float* scales, hipStream_t stream) {
  const int32_t nb = (N + block - 1) / block;
  const int64_t grid = (int64_t)B * H * nb;
  if (grid > 0x7fffffffLL) return fail(RADIAL_ESHAPE, "B*H*n_blocks is too large for one launch");
  quantize_fp8_kernel<<<dim3((unsigned)grid), dim3(256), 0, stream>>>(x, codes, scales, H, N, Dh, block, nb);
  RADIAL_HIP_TRY(hipGetLastError());
  return RADIAL_OK;
}

int launch_fwd_fp8(const Fp8FwdArgs& a, hipStream_t stream) {
  const int64_t grid = 8LL * a.B * a.H * a.max_slice;
  if (grid > 0x7fffffffLL) return fail(RADIAL_ESHAPE, "B*H*n_blocks is too large for one launch");
  if (grid == 0) return RADIAL_OK;
  radial_fwd_fp8_kernel<<<dim3((unsigned)grid), dim3(kThreads), 0, stream>>>(a);
  RADIAL_HIP_TRY(hipGetLastError());
  return RADIAL_OK;
}

}  // namespace radial
