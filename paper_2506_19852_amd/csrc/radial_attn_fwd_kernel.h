// Block-sparse attention forward kernel for gfx950 (template; instantiated by radial_attn_fwd.hip and,
// with per-workgroup trace records, by radial_diag.hip): Eq. 2 of the paper evaluated only on the key
// blocks that the block list names (Eq. 1 when the list names all of them).
//
// One workgroup = one (batch, head, query block).  Wave w owns 32 query rows.  Everything
// that belongs to query row r lives in lanes r and r+32 of that wave, because both products
// are computed transposed on v_mfma_f32_32x32x16_bf16:
//     S^T[key, q] = K[key, :] . Q[q, :]      A = K tile (LDS),     B = Q^T (registers)
//     O^T[d,   q] = V^T[d, key] . P^T[key, q] A = V^T (LDS, transposing read), B = P^T (registers)
// The accumulator layout of the first product (column = lane%32, 16 rows per lane) is, 8
// rows at a time, exactly the B-operand layout of the second one, so P never leaves
// registers, row maxima and sums are in-lane reductions plus one exchange with lane^32, and
// the running rescale of O is a per-lane multiply.
//
// Key blocks are walked in stages of 64 keys (32 for head dimension 128 with 64-token blocks).  The K and V rows of a stage are copied
// HBM -> LDS by global_load_lds (no register staging) into one of two LDS stage buffers; the
// copy of stage u+1 is issued right after the barrier that opens stage u, so it overlaps
// the whole of stage u's arithmetic and a stage needs exactly one barrier.  The copies are
// issued from inline assembly and waited for explicitly (s_waitcnt vmcnt(0) before that
// barrier): otherwise the compiler orders every LDS read after all outstanding copies.
// 16-byte pieces are XOR-swizzled inside 256-byte LDS lines so that the 128-bit K reads and
// the 64-bit transposing V reads are bank-conflict free.
#pragma once

#include <type_traits>

#include "radial_internal.h"
#include "radial_tile.h"

namespace radial {
namespace fwd {

template <int D, int BLK>
struct Tile {
  // Keys per pipeline stage.  Head dimension 128 with 64-token blocks walks half-size stages: two
  // 64-key stage buffers (64 KiB) per 2-wave workgroup would leave a compute unit with 4 waves.
  static constexpr int kStageKeys = (D == 128 && BLK == 64) ? 32 : 64;
  static constexpr int kWaves = BLK / 32;          // one wave per 32 query rows
  static constexpr int kThreads = 64 * kWaves;
  static constexpr int kPiecesPerRow = D / 8;      // 16-byte pieces per K/V row
  static constexpr int kSubs = BLK / kStageKeys;   // stages per listed key block
  static constexpr int kStageBytes = kStageKeys * D * 2;            // one K (or V) stage tile
  static constexpr int kLoadsPerWave = kStageBytes / 1024 / kWaves; // 1 KiB copies per wave per tile
  static constexpr int kSteps = D / 16;            // MFMA k-steps of the S product
  static constexpr int kKeyTiles = kStageKeys / 32;
  static constexpr int kDTiles = D / 32;           // 32-wide d tiles of O
  // MFMAs of the first product per copy of the next stage (copies are spread over that product)
  static constexpr int kCopyEvery = (kKeyTiles * kSteps) / (2 * kLoadsPerWave);
  static_assert(kCopyEvery >= 1, "more copies than MFMAs in the first product");
};

// Swizzle key of a 256-byte LDS line (16 pieces of 16 bytes); pieces move inside their line only.
template <int D, bool kIsV>
__device__ __forceinline__ int swizzle_key(int line) {
  if (kIsV) return D == 128 ? ((line & 3) << 2) : ((line & 1) << 2);
  return D == 128 ? (line & 15) : (line & 7);
}

// LDS byte offset of 16-byte piece p of tile row r.
template <int D, bool kIsV>
__device__ __forceinline__ int piece_offset(int r, int p) {
  const int lin = r * (D / 8) + p;
  const int line = lin >> 4, slot = lin & 15;
  return (line << 8) + ((slot ^ swizzle_key<D, kIsV>(line)) << 4);
}

// kExact: apply the token-level rule of the radial mask inside the listed blocks.
// kTrace: also record begin, end and hardware ids of the workgroup (diagnostics build of the kernel;
// the library's radial_attn_fwd launches kTrace = false, which carries none of it).
template <int D, int BLK, bool kExact, bool kTrace>
// Two waves per SIMD: two 4-wave workgroups per compute unit (BLK = 128) or four 2-wave ones (BLK = 64).
__global__ void __launch_bounds__(2 * BLK, 2) radial_fwd_kernel(const FwdArgs a) {
  using T = Tile<D, BLK>;
  // [stage buffer][K, V][T::kStageKeys x D bf16]
  __shared__ __attribute__((aligned(1024))) char lds[2 * 2 * T::kStageBytes];
  const uint32_t lds_base = lds_address(lds);

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lq = lane & 31;   // query column / K row inside a 32-tile
  const int g = lane >> 5;    // which half of the 16-wide MFMA k-slice this lane feeds

  // Workgroup -> work item.  Consecutive workgroup ids go to different XCDs.  The query blocks are
  // cut into 8 slices of equal list weight; for head bh, XCD x takes slice (x + bh) mod 8 and the
  // XCDs move from head to head together, so all of them work on the same head at the same time
  // (its K/V stay in the shared last-level cache), neighbouring workgroups of an XCD share K/V
  // tiles in that XCD's L2, and every XCD gets every slice equally often (slices of equal weight
  // do not take exactly equal time).
  const uint64_t t_begin = kTrace ? __builtin_amdgcn_s_memrealtime() : 0;
  const int32_t xcd = blockIdx.x & 7;
  const int64_t idx = blockIdx.x >> 3;
  const int32_t bh = (int32_t)(idx / a.max_slice);
  const int32_t pos = (int32_t)(idx % a.max_slice);
  const int32_t sl = (xcd + bh) & 7;
  const int32_t s0 = a.slice[sl];
  if (pos >= a.slice[sl + 1] - s0) return;
  const int32_t qb = s0 + pos;
  const int32_t b = bh / a.H, h = bh % a.H;

  const __bf16* qp = (const __bf16*)a.q.ptr + (int64_t)b * a.q.sb + (int64_t)h * a.q.sh;
  const __bf16* kp = (const __bf16*)a.k.ptr + (int64_t)b * a.k.sb + (int64_t)h * a.k.sh;
  const __bf16* vp = (const __bf16*)a.v.ptr + (int64_t)b * a.v.sb + (int64_t)h * a.v.sh;
  __bf16* op = (__bf16*)a.o.ptr + (int64_t)b * a.o.sb + (int64_t)h * a.o.sh;

  const int32_t list_lo = __builtin_amdgcn_readfirstlane(a.row_ptr[qb]);
  const int32_t n_list = __builtin_amdgcn_readfirstlane(a.row_ptr[qb + 1]) - list_lo;
  const int32_t n_stage = n_list * T::kSubs;
  const int32_t q_row = qb * BLK + wave * 32 + lq;
  const bool q_ok = q_row < a.N;

  // Q^T fragments: for k-step t this lane holds Q[q_row, 16t + 8g .. +7].
  bf16x8 qf[T::kSteps];
  {
    const __bf16* src = qp + (int64_t)(q_ok ? q_row : a.N - 1) * a.q.sn + 8 * g;
#pragma unroll
    for (int t = 0; t < T::kSteps; ++t) {
      u32x4 raw = *(const u32x4*)(src + 16 * t);
      if (!q_ok) raw = u32x4{0u, 0u, 0u, 0u};
      qf[t] = __builtin_bit_cast(bf16x8, raw);
    }
  }

  // The list entries of this row, 64 at a time in one register per lane; cvec is the chunk
  // being walked, nvec the one after it.
  const int32_t* cols = a.col_idx + list_lo;
  int32_t cvec = lane < n_list ? cols[lane] : 0;
  int32_t nvec = 64 + lane < n_list ? cols[64 + lane] : 0;
  // token rule: this lane's query as (frame, position), and the same for the first token of
  // every listed key block (one division per lane per 64 entries)
  StagePos q_at = {0, 0}, cvec_at = {0, 0};
  if (kExact) {
    q_at = block_pos(q_ok ? q_row : a.N - 1, a.rule.s);
    cvec_at = block_pos(cvec * BLK, a.rule.s);
  }

  // Which piece of a stage tile each of this lane's copies fetches (fixed for the kernel),
  // as a byte offset from the first row of the tile.
  int32_t krow[T::kLoadsPerWave], kcol[T::kLoadsPerWave], vrow_[T::kLoadsPerWave], vcol[T::kLoadsPerWave];
  uint32_t koff[T::kLoadsPerWave], voff[T::kLoadsPerWave];
#pragma unroll
  for (int i = 0; i < T::kLoadsPerWave; ++i) {
    const int lin = (wave * T::kLoadsPerWave + i) * 64 + lane;  // LDS piece this lane fills
    const int line = lin >> 4, slot = lin & 15;
    const int ksrc = (line << 4) + (slot ^ swizzle_key<D, false>(line));
    const int vsrc = (line << 4) + (slot ^ swizzle_key<D, true>(line));
    krow[i] = ksrc / T::kPiecesPerRow;
    kcol[i] = (ksrc % T::kPiecesPerRow) * 8;
    vrow_[i] = vsrc / T::kPiecesPerRow;
    vcol[i] = (vsrc % T::kPiecesPerRow) * 8;
    koff[i] = (uint32_t)(krow[i] * (int32_t)a.k.sn + kcol[i]) * 2u;
    voff[i] = (uint32_t)(vrow_[i] * (int32_t)a.v.sn + vcol[i]) * 2u;
  }
  // Copies the 64 K rows and V rows starting at key `key0` into stage buffer `buf`.
  // Rows past N-1 are clamped to N-1; their scores are masked before the softmax.
  auto issue_stage = [&](int32_t key0, int buf) {
    const uint32_t kdst = lds_base + buf * 2 * T::kStageBytes + wave * T::kLoadsPerWave * 1024;
    const uint32_t vdst = kdst + T::kStageBytes;
    const __bf16* kbase = kp + (int64_t)key0 * a.k.sn;  // wave-uniform
    const __bf16* vbase = vp + (int64_t)key0 * a.v.sn;
    if (key0 + T::kStageKeys <= a.N) {
#pragma unroll
      for (int i = 0; i < T::kLoadsPerWave; ++i) copy16_to_lds_sv(kbase, koff[i], kdst + i * 1024);
#pragma unroll
      for (int i = 0; i < T::kLoadsPerWave; ++i) copy16_to_lds_sv(vbase, voff[i], vdst + i * 1024);
    } else {  // ragged end of the sequence
      const int32_t last = a.N - 1 - key0;  // >= 0: a listed block starts below N; a stage past N reads row N-1
#pragma unroll
      for (int i = 0; i < T::kLoadsPerWave; ++i) {
        const int32_t r = krow[i] < last ? krow[i] : last;
        copy16_to_lds(kp + ((int64_t)key0 + r) * a.k.sn + kcol[i], kdst + i * 1024);
      }
#pragma unroll
      for (int i = 0; i < T::kLoadsPerWave; ++i) {
        const int32_t r = vrow_[i] < last ? vrow_[i] : last;
        copy16_to_lds(vp + ((int64_t)key0 + r) * a.v.sn + vcol[i], vdst + i * 1024);
      }
    }
  };

  f32x16 o[T::kDTiles];
#pragma unroll
  for (int i = 0; i < T::kDTiles; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) o[i][e] = 0.f;
  float m_run = -INFINITY;  // running row maximum of the raw (unscaled) scores
  float l_run = 0.f;        // this lane's share of the running row sum
  const float c = a.scale * 1.4426950408889634f;  // exp(scale*x) = exp2(c*x)

  int32_t key0 = 0;  // first key of the stage about to be computed
  StagePos k_at = {0, 0}, k_at_next = {0, 0};  // its (frame, position), and the next stage's
  if (n_stage > 0) {
    key0 = __builtin_amdgcn_readlane(cvec, 0) * BLK;
    if (kExact) k_at = stage_pos(cvec_at, 0, 0, a.rule.s);
    issue_stage(key0, 0);
  }

  // One stage: scores of 64 keys, online softmax, O update.  spread_lanes (all or none): also issue this
  // wave's copies of the next stage between the MFMAs of the first product.
  auto stage_body = [&](int buf, int32_t key0, int32_t key0_next, const StageRule& vis, uint64_t spread_lanes) __attribute__((always_inline)) {
    const uint32_t kdst_next = lds_base + (buf ^ 1) * 2 * T::kStageBytes + wave * T::kLoadsPerWave * 1024;
    const uint32_t vdst_next = kdst_next + T::kStageBytes;
    const __bf16* kbase_next = kp + (int64_t)key0_next * a.k.sn;  // wave-uniform
    const __bf16* vbase_next = vp + (int64_t)key0_next * a.v.sn;
    const char* lds_k = lds + buf * 2 * T::kStageBytes;
    const char* lds_v = lds_k + T::kStageBytes;

    // ---- S^T = K Q^T -------------------------------------------------------------------
    f32x16 s[T::kKeyTiles];
#pragma unroll
    for (int kt = 0; kt < T::kKeyTiles; ++kt) {
#pragma unroll
      for (int e = 0; e < 16; ++e) s[kt][e] = 0.f;
#pragma unroll
      for (int t = 0; t < T::kSteps; ++t) {
        const bf16x8 kf = *lds_cast<const bf16x8>(lds_k + piece_offset<D, false>(kt * 32 + lq, 2 * t + g));
        s[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[t], s[kt], 0, 0, 0);
        {  // one copy of stage u+1 every kCopyEvery MFMAs
          const int m = kt * T::kSteps + t + 1;
          const int j = m / T::kCopyEvery - 1;
          if (m % T::kCopyEvery == 0 && j < T::kLoadsPerWave)
            copy16_to_lds_sv_masked(kbase_next, koff[j], kdst_next + j * 1024, spread_lanes);
          else if (m % T::kCopyEvery == 0 && j < 2 * T::kLoadsPerWave)
            copy16_to_lds_sv_masked(vbase_next, voff[j - T::kLoadsPerWave], vdst_next + (j - T::kLoadsPerWave) * 1024, spread_lanes);
        }
      }
    }

    // ---- online softmax ------------------------------------------------------------------
    // s[kt][e] belongs to key key0 + 32kt + 8(e/4) + 4g + e%4 and query q_row.  Keys >= N do not
    // exist; under the token rule some keys are hidden from this lane's query.
    if (key0 + T::kStageKeys > a.N || (kExact && vis.partial)) {
      uint64_t seen = stage_prefix(a.N - key0);
      if (kExact) seen &= vis.visible_mask();
      const uint32_t hidden = ~lane_element_bits(seen, g);
      if (__builtin_amdgcn_ballot_w64(hidden != 0u) != 0) {
#pragma unroll
        for (int kt = 0; kt < T::kKeyTiles; ++kt)
#pragma unroll
          for (int e = 0; e < 16; ++e)
            if ((hidden >> (16 * kt + e)) & 1u) s[kt][e] = -INFINITY;
      }
    }
    float mx = s[0][0];
#pragma unroll
    for (int kt = 0; kt < T::kKeyTiles; ++kt)
#pragma unroll
      for (int e = 0; e < 16; ++e) mx = fmaxf(mx, s[kt][e]);
    mx = max_with_other_half(mx);  // the other 32 keys of the row's stage
    // A stage that lies entirely past N (second half of a ragged last block) has mx = -inf.
    const float m_new = fmaxf(m_run, mx);
    if (__builtin_amdgcn_ballot_w64(m_new > m_run) != 0) {  // some row of this wave got a new maximum
      const float alpha = m_new > m_run ? __builtin_amdgcn_exp2f((m_run - m_new) * c) : 1.f;
      l_run *= alpha;
#pragma unroll
      for (int i = 0; i < T::kDTiles; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[i][e] *= alpha;
      m_run = m_new;
    }
    const float mc = m_run == -INFINITY ? 0.f : m_run * c;
    float psum = 0.f;
    uint32_t pk[T::kKeyTiles][8];  // P^T as bf16 pairs: B operands of the second product
#pragma unroll
    for (int kt = 0; kt < T::kKeyTiles; ++kt)
#pragma unroll
      for (int e = 0; e < 16; e += 2) {
        const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kt][e], c, -mc));
        const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kt][e + 1], c, -mc));
        psum += p0 + p1;
        pk[kt][e >> 1] = pack_bf16(p0, p1);
      }
    l_run += psum;

    // ---- O^T += V^T P^T --------------------------------------------------------------------
#pragma unroll
    for (int kt = 0; kt < T::kKeyTiles; ++kt)
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const u32x4 praw = {pk[kt][4 * t], pk[kt][4 * t + 1], pk[kt][4 * t + 2], pk[kt][4 * t + 3]};
        const bf16x8 pf = __builtin_bit_cast(bf16x8, praw);
#pragma unroll
        for (int dt = 0; dt < T::kDTiles; ++dt) {
          // Lanes 0-15 / 16-31 / 32-47 / 48-63 each transpose a 4-key x 16-d patch: lane i of
          // a group reads 4 d-contiguous values of key i/4 and receives the 4 keys of d column i.
          const int i16 = lane & 15;
          const int vrow = kt * 32 + 16 * t + 4 * g + (i16 >> 2);
          const int dcol = 32 * dt + 16 * ((lane >> 4) & 1) + 4 * (i16 & 3);
          const int off0 = piece_offset<D, true>(vrow, dcol >> 3) + ((dcol & 7) << 1);
          const int off1 = piece_offset<D, true>(vrow + 8, dcol >> 3) + ((dcol & 7) << 1);
          const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(lds_cast<s16x4>(lds_v + off0));
          const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(lds_cast<s16x4>(lds_v + off1));
          const u32x2 a0 = __builtin_bit_cast(u32x2, v0), a1 = __builtin_bit_cast(u32x2, v1);
          const u32x4 vraw = {a0[0], a0[1], a1[0], a1[1]};
          o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vraw), pf, o[dt], 0, 0, 0);
        }
      }
  };

  // Two stages per trip, so that the stage buffer of each half is a compile-time constant and the
  // LDS addresses of its reads are immediates.
  auto one_stage = [&](int32_t u, auto buf_c) __attribute__((always_inline)) {
    constexpr int buf = decltype(buf_c)::value;
    // First key of stage u+1.
    int32_t key0_next = 0;
    const bool has_next = u + 1 < n_stage;
    if (has_next) {
      const int32_t e1 = (u + 1) / T::kSubs;
      if ((u + 1) % T::kSubs == 0 && (e1 & 63) == 0) {  // entering the next chunk of the list
        cvec = nvec;
        nvec = e1 + 64 + lane < n_list ? cols[e1 + 64 + lane] : 0;
        if (kExact) cvec_at = block_pos(cvec * BLK, a.rule.s);
      }
      key0_next = __builtin_amdgcn_readlane(cvec, e1 & 63) * BLK + ((u + 1) % T::kSubs) * T::kStageKeys;
      if (kExact) k_at_next = stage_pos(cvec_at, e1 & 63, ((u + 1) % T::kSubs) * T::kStageKeys, a.rule.s);
    }

    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this wave's copies of stage u have landed
    __syncthreads();                                  // ... and everyone's; stage u-1 is fully consumed

    StageRule vis = {};
    bool skip = false;
    if (kExact) {
      vis = stage_rule<T::kStageKeys>(a.rule, q_at, k_at, true);
      skip = vis.none;  // nothing in this stage for any row of this wave
    }
    // The copies of stage u+1 are spread over the first product of stage u (a burst of copies
    // would hold the wave at the memory pipeline before it reaches its first MFMA); only a
    // ragged next stage, or a stage this wave skips, issues them in one go.
    const bool spread = has_next && !skip && key0_next + T::kStageKeys <= a.N;
    if (has_next && !spread) issue_stage(key0_next, buf ^ 1);
    if (!skip) {
      const uint32_t on = __builtin_amdgcn_readfirstlane(spread ? ~0u : 0u);  // wave-uniform by construction
      stage_body(buf, key0, spread ? key0_next : key0, vis, ((uint64_t)on << 32) | on);
    }
    key0 = key0_next;
    k_at = k_at_next;
  };
  for (int32_t u = 0; u < n_stage; u += 2) {
    one_stage(u, std::integral_constant<int, 0>{});
    if (u + 1 < n_stage) one_stage(u + 1, std::integral_constant<int, 1>{});
  }

  // ---- epilogue: O / l, LSE ----------------------------------------------------------------
  const float l_tot = l_run + __shfl_xor(l_run, 32);
  const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
  if (q_ok) {
    __bf16* dst = op + (int64_t)q_row * a.o.sn;
#pragma unroll
    for (int dt = 0; dt < T::kDTiles; ++dt)
#pragma unroll
      for (int e4 = 0; e4 < 4; ++e4) {
        // o[dt][4*e4 + x] is d = 32dt + 8*e4 + 4g + x
        u32x2 w;
        w[0] = pack_bf16(o[dt][4 * e4] * inv, o[dt][4 * e4 + 1] * inv);
        w[1] = pack_bf16(o[dt][4 * e4 + 2] * inv, o[dt][4 * e4 + 3] * inv);
        *(u32x2*)(dst + 32 * dt + 8 * e4 + 4 * g) = w;
      }
    if (a.lse && g == 0) {
      const int64_t idx = ((int64_t)b * a.H + h) * a.N + q_row;
      a.lse[idx] = l_tot > 0.f ? m_run * a.scale + __logf(l_tot) : -INFINITY;
    }
  }
  if (kTrace && a.wg_trace != nullptr && threadIdx.x == 0) {
    // hardware id registers: which XCD, shader engine and compute unit this workgroup ran on
    constexpr int kHwId = 4, kXccId = 20, kAllBits = 31 << 11;
    const uint64_t where = ((uint64_t)__builtin_amdgcn_s_getreg(kXccId | kAllBits) << 32) | (uint32_t)__builtin_amdgcn_s_getreg(kHwId | kAllBits);
    uint64_t* rec = a.wg_trace + 3 * (int64_t)blockIdx.x;
    rec[0] = t_begin;
    rec[1] = __builtin_amdgcn_s_memrealtime();
    rec[2] = where;
  }
}

// Launches the kernel instance for (D, block, token rule); kTrace selects the diagnostics build.
template <int D, int BLK, bool kTrace>
int launch(const FwdArgs& a, hipStream_t stream) {
  const int64_t grid = 8LL * a.B * a.H * a.max_slice;
  if (grid > 0x7fffffffLL) return fail(RADIAL_ESHAPE, "B*H*n_blocks is too large for one launch");
  if (grid == 0) return RADIAL_OK;
  if (a.rule.exact)
    radial_fwd_kernel<D, BLK, true, kTrace><<<dim3((unsigned)grid), dim3(Tile<D, BLK>::kThreads), 0, stream>>>(a);
  else
    radial_fwd_kernel<D, BLK, false, kTrace><<<dim3((unsigned)grid), dim3(Tile<D, BLK>::kThreads), 0, stream>>>(a);
  RADIAL_HIP_TRY(hipGetLastError());
  return RADIAL_OK;
}

template <bool kTrace>
int launch_any(int D, int block, const FwdArgs& a, hipStream_t stream) {
  if (D == 128 && block == 128) return launch<128, 128, kTrace>(a, stream);
  if (D == 64 && block == 128) return launch<64, 128, kTrace>(a, stream);
  if (D == 128 && block == 64) return launch<128, 64, kTrace>(a, stream);
  if (D == 64 && block == 64) return launch<64, 64, kTrace>(a, stream);
  return fail(RADIAL_EUNSUPPORTED, "head dimension %d with block %d is not supported", D, block);
}

}  // namespace fwd
}  // namespace radial
