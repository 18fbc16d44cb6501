// Block-sparse attention backward for gfx950: the gradient of Eq. 2 of the paper restricted to
// the listed block pairs,
//     P = exp(scale*Q K^T - LSE),  dV = P^T dO,  dP = dO V^T,  delta = rowsum(dO * O),
//     dS = P * (dP - delta),       dQ = scale * dS K,          dK = scale * dS^T Q.
//
// Three kernels, no atomics (results are reproducible run to run):
//   prepare : delta[b,h,q] = sum_d dO*O;
//   dkdv    : one workgroup per (batch, head, key block) walks the transposed list (the query
//             blocks that list this key block) in stages of 64 query rows.  Wave w owns 32
//             keys; its K and V rows stay in registers, dK^T and dV^T accumulate in registers
//             (column = key = lane%32).  S and dP are computed with query rows as MFMA rows
//             so that P and dS come out with keys across lanes: 8 accumulator rows at a time
//             they are the B operands of dV^T += dO^T P and dK^T += Q^T dS, whose A operands
//             are transposing LDS reads of the dO and Q stage tiles;
//   dq      : one workgroup per (batch, head, query block) walks the row list in stages of 64
//             keys, like the forward kernel: wave w owns 32 query rows whose Q and dO rows stay
//             in registers; S^T = K Q^T and dP^T = V dO^T come out with queries across lanes,
//             LSE and delta are per-lane scalars, and dS^T feeds dQ^T += K^T dS^T from registers
//             (A operand: transposing LDS reads of the K stage tile).  S and dP are recomputed
//             here (7 products in total instead of 5), which is cheaper than pushing every
//             listed pair's 64 KiB of dQ partial sums through memory atomics.
// Stage tiles are copied HBM -> LDS by global_load_lds, double buffered, one stage ahead.
#include <atomic>

#include "radial_internal.h"
#include "radial_tile.h"

namespace radial {
namespace {

constexpr int kStageQ = 64;  // query rows per pipeline stage
constexpr float kLog2e = 1.4426950408889634f;

template <int D, int BLK>
struct BwdTile {
  static constexpr int kWaves = BLK / 32;  // one wave per 32 keys
  static constexpr int kThreads = 64 * kWaves;
  static constexpr int kSubs = BLK / kStageQ;  // stages per listed query block
  static constexpr int kSteps = D / 16;
  static constexpr int kDTiles = D / 32;
  static constexpr int kQBytes = kStageQ * D * 2;        // Q or dO stage tile
  static constexpr int kStatBytes = 2 * kStageQ * 4;     // LSE and delta of a stage
  static constexpr int kStageBytes = 2 * kQBytes + kStatBytes;
  static constexpr int kLdsBytes = 2 * kStageBytes;
  static constexpr int kQLoadsPerWave = kQBytes / 1024 / kWaves;
};

template <int D>
__global__ void __launch_bounds__(256) bwd_prepare_kernel(const BwdArgs a) {
  constexpr int kLanesPerRow = D / 8;
  constexpr int kRowsPerBlock = 256 / kLanesPerRow;
  const int64_t rows = (int64_t)a.B * a.H * a.N;
  const int64_t row = (int64_t)blockIdx.x * kRowsPerBlock + threadIdx.x / kLanesPerRow;
  const int piece = threadIdx.x % kLanesPerRow;
  float sum = 0.f;
  if (row < rows) {
    const int32_t q = (int32_t)(row % a.N);
    const int32_t bh = (int32_t)(row / a.N);
    const int32_t b = bh / a.H, h = bh % a.H;
    const __bf16* o = (const __bf16*)a.o.ptr + (int64_t)b * a.o.sb + (int64_t)h * a.o.sh + (int64_t)q * a.o.sn + piece * 8;
    const __bf16* g = (const __bf16*)a.dout.ptr + (int64_t)b * a.dout.sb + (int64_t)h * a.dout.sh + (int64_t)q * a.dout.sn + piece * 8;
    const bf16x8 ov = *(const bf16x8*)o;
    const bf16x8 gv = *(const bf16x8*)g;
#pragma unroll
    for (int i = 0; i < 8; ++i) sum += (float)ov[i] * (float)gv[i];
  }
#pragma unroll
  for (int off = kLanesPerRow / 2; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
  if (row < rows && piece == 0) a.delta[row] = sum;
}

// acc (+)= a * b with the accumulator in ordinary vector registers.  In a kernel that uses both
// register files the compiler places every MFMA result in the accumulation file; S and dP are
// consumed by vector instructions, which cannot read that file, so each of their 64 values per stage
// would be copied out one register at a time (a third of the kernel's vector instructions).
// The instruction is opaque to the compiler's hazard tracking.  What the compiler would guarantee
// is arranged here or checked on the compiled code by tests/test_kernel_asm.py:
//   - the result registers of the first k-step overlap no operand (early clobber);
//   - no vector instruction writes an operand within two wait states before the MFMA (checked);
//   - before a vector instruction reads or writes acc the caller waits with mfma_results_settle(),
//     and nothing else names acc in between (checked);
//   - a second MFMA on the same accumulator follows after one other MFMA at the earliest.
__device__ __forceinline__ void mfma32_vgpr_first(f32x16& acc, bf16x8 a, bf16x8 b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(acc) : "v"(a), "v"(b));
}
__device__ __forceinline__ void mfma32_vgpr(f32x16& acc, bf16x8 a, bf16x8 b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b));
}
// 16 wait states: more than the 11 an 8-pass MFMA needs before a vector instruction touches its result.
// The accumulators are operands so that every later use of them stays behind the wait.
__device__ __forceinline__ void mfma_results_settle(f32x16& acc0, f32x16& acc1) {
  asm volatile("s_nop 15" : "+v"(acc0), "+v"(acc1));
}

// kExact (all three kernels' callers): apply the token-level rule inside the listed blocks.
template <int D, int BLK, bool kExact>
__global__ void __launch_bounds__(2 * BLK, 1) radial_bwd_dkdv_kernel(const BwdArgs a) {
  using T = BwdTile<D, BLK>;
  using QT = SwzTile<D>;  // Q, dO tiles: rows of D elements
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const uint32_t lds_base = lds_address(lds);

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lq = lane & 31;
  const int g = lane >> 5;
  const int i16 = lane & 15;
  const int half16 = (lane >> 4) & 1;

  // work item: XCD x owns the key blocks [slice_t[x], slice_t[x+1]) of every (batch, head)
  const int32_t xcd = blockIdx.x & 7;
  const int32_t s0 = a.slice_t[xcd];
  const int32_t slice_len = a.slice_t[xcd + 1] - s0;
  const int64_t idx = blockIdx.x >> 3;
  if (slice_len <= 0 || idx >= (int64_t)slice_len * a.B * a.H) return;
  const int32_t bh = (int32_t)(idx / slice_len);
  const int32_t kb = s0 + (int32_t)(idx % slice_len);
  const int32_t b = bh / a.H, h = bh % a.H;

  const __bf16* qp = (const __bf16*)a.q.ptr + (int64_t)b * a.q.sb + (int64_t)h * a.q.sh;
  const __bf16* kp = (const __bf16*)a.k.ptr + (int64_t)b * a.k.sb + (int64_t)h * a.k.sh;
  const __bf16* vp = (const __bf16*)a.v.ptr + (int64_t)b * a.v.sb + (int64_t)h * a.v.sh;
  const __bf16* gp = (const __bf16*)a.dout.ptr + (int64_t)b * a.dout.sb + (int64_t)h * a.dout.sh;
  const float* lsep = a.lse + (int64_t)bh * a.N;
  const float* deltap = a.delta + (int64_t)bh * a.N;

  const int32_t list_lo = __builtin_amdgcn_readfirstlane(a.col_ptr[kb]);
  const int32_t n_list = __builtin_amdgcn_readfirstlane(a.col_ptr[kb + 1]) - list_lo;
  const int32_t n_stage = n_list * T::kSubs;
  const int32_t key_row = kb * BLK + wave * 32 + lq;
  const bool key_ok = key_row < a.N;

  // K and V rows of this lane's key: B operands of S = Q K^T and dP = dO V^T.
  bf16x8 kf[T::kSteps], vf[T::kSteps];
  {
    const int64_t r = key_ok ? key_row : a.N - 1;
    const __bf16* ks = kp + r * a.k.sn + 8 * g;
    const __bf16* vs = vp + r * a.v.sn + 8 * g;
#pragma unroll
    for (int t = 0; t < T::kSteps; ++t) {
      u32x4 kr = *(const u32x4*)(ks + 16 * t), vr = *(const u32x4*)(vs + 16 * t);
      if (!key_ok) kr = vr = u32x4{0u, 0u, 0u, 0u};
      kf[t] = __builtin_bit_cast(bf16x8, kr);
      vf[t] = __builtin_bit_cast(bf16x8, vr);
    }
  }

  const int32_t* rows_list = a.row_idx + list_lo;
  int32_t cvec = lane < n_list ? rows_list[lane] : 0;
  int32_t nvec = 64 + lane < n_list ? rows_list[64 + lane] : 0;
  // token rule: (frame, position) of this lane's key and of every listed query block's first row
  StagePos key_at = {0, 0}, cvec_at = {0, 0};
  if (kExact) {
    key_at = block_pos(key_ok ? key_row : a.N - 1, a.rule.s);
    cvec_at = block_pos(cvec * BLK, a.rule.s);
  }

  int32_t srow[T::kQLoadsPerWave], scol[T::kQLoadsPerWave];
#pragma unroll
  for (int i = 0; i < T::kQLoadsPerWave; ++i) QT::source_of((wave * T::kQLoadsPerWave + i) * 64 + lane, srow[i], scol[i]);

  uint32_t qoff[T::kQLoadsPerWave], goff[T::kQLoadsPerWave];  // byte offsets from the stage's first row
#pragma unroll
  for (int i = 0; i < T::kQLoadsPerWave; ++i) {
    qoff[i] = (uint32_t)(srow[i] * (int32_t)a.q.sn + scol[i]) * 2u;
    goff[i] = (uint32_t)(srow[i] * (int32_t)a.dout.sn + scol[i]) * 2u;
  }
  // Copies Q, dO (64 rows from q0) and their LSE / delta into stage buffer `buf`, all at once
  // (first stage, ragged stages; rows past N-1 are clamped to N-1).
  auto issue_stage = [&](int32_t q0, int buf) {
    const uint32_t qdst = lds_base + buf * T::kStageBytes + wave * T::kQLoadsPerWave * 1024;
    const uint32_t gdst = qdst + T::kQBytes;
#pragma unroll
    for (int i = 0; i < T::kQLoadsPerWave; ++i) {
      int32_t r = q0 + srow[i];
      r = r < a.N ? r : a.N - 1;
      copy16_to_lds(qp + (int64_t)r * a.q.sn + scol[i], qdst + i * 1024);
      copy16_to_lds(gp + (int64_t)r * a.dout.sn + scol[i], gdst + i * 1024);
    }
    if (wave < 2) {
      int32_t r = q0 + lane;
      r = r < a.N ? r : a.N - 1;
      const uint32_t sdst = lds_base + buf * T::kStageBytes + 2 * T::kQBytes + wave * kStageQ * 4;
      copy4_to_lds((wave == 0 ? lsep : deltap) + r, sdst);
    }
  };

  f32x16 dk[T::kDTiles], dv[T::kDTiles];
#pragma unroll
  for (int i = 0; i < T::kDTiles; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) dk[i][e] = dv[i][e] = 0.f;
  const float c = a.scale * kLog2e;

  int32_t q0 = 0;
  StagePos q_at = {0, 0}, q_at_next = {0, 0};
  if (n_stage > 0) {
    q0 = __builtin_amdgcn_readlane(cvec, 0) * BLK;
    if (kExact) q_at = stage_pos(cvec_at, 0, 0, a.rule.s);
    issue_stage(q0, 0);
  }

  for (int32_t u = 0; u < n_stage; ++u) {
    const int buf = u & 1;
    int32_t q0_next = 0;
    const bool has_next = u + 1 < n_stage;
    if (has_next) {
      const int32_t e1 = (u + 1) / T::kSubs;
      if ((u + 1) % T::kSubs == 0 && (e1 & 63) == 0) {
        cvec = nvec;
        nvec = e1 + 64 + lane < n_list ? rows_list[e1 + 64 + lane] : 0;
        if (kExact) cvec_at = block_pos(cvec * BLK, a.rule.s);
      }
      q0_next = __builtin_amdgcn_readlane(cvec, e1 & 63) * BLK + ((u + 1) % T::kSubs) * kStageQ;
      if (kExact) q_at_next = stage_pos(cvec_at, e1 & 63, ((u + 1) % T::kSubs) * kStageQ, a.rule.s);
    }

    wait_all_copies();  // stage u has landed
    __syncthreads();    // for every wave; stage u-1 is finished
    // The copies of a full next stage are spread over the first MFMAs of this one (see below);
    // a ragged one is issued at once.
    const bool spread_next = has_next && q0_next + kStageQ <= a.N;
    if (has_next && !spread_next) issue_stage(q0_next, buf ^ 1);

    const char* sq = lds + buf * T::kStageBytes;
    const char* sg = sq + T::kQBytes;
    const char* st = sg + T::kQBytes;  // 64 x LSE then 64 x delta
    const bool ragged_q = q0 + kStageQ > a.N;
    StageRule vis = {};
    if (kExact) vis = stage_rule(a.rule, key_at, q_at, false);  // which of the stage's queries see this lane's key
    uint32_t hidden = 0u;
    if (ragged_q || (kExact && vis.partial)) {  // query rows past N, rows the token rule hides from this key
      uint64_t seen = stage_prefix(a.N - q0);
      if (kExact) seen &= vis.visible_mask();
      hidden = ~lane_element_bits(seen, g);
    }
    const bool any_hidden = __builtin_amdgcn_ballot_w64(hidden != 0u) != 0;
    // this wave's copies of the next stage, one or two per k-step of phase A
    const uint32_t on = __builtin_amdgcn_readfirstlane(spread_next ? ~0u : 0u);
    const uint64_t copy_lanes = ((uint64_t)on << 32) | on;
    const int32_t q_src = spread_next ? q0_next : q0;  // any valid row when the copies are switched off
    const __bf16* qbase_next = qp + (int64_t)q_src * a.q.sn;
    const __bf16* gbase_next = gp + (int64_t)q_src * a.dout.sn;
    const uint32_t qdst_next = lds_base + (buf ^ 1) * T::kStageBytes + wave * T::kQLoadsPerWave * 1024;
    const uint32_t gdst_next = qdst_next + T::kQBytes;
    auto spread_copy = [&](int j) {  // j = 0 .. 2 * kQLoadsPerWave: Q pieces, dO pieces, LSE/delta
      if (j < T::kQLoadsPerWave) {
        copy16_to_lds_sv_masked(qbase_next, qoff[j], qdst_next + j * 1024, copy_lanes);
      } else if (j < 2 * T::kQLoadsPerWave) {
        copy16_to_lds_sv_masked(gbase_next, goff[j - T::kQLoadsPerWave], gdst_next + (j - T::kQLoadsPerWave) * 1024, copy_lanes);
      } else if (j == 2 * T::kQLoadsPerWave) {
        const uint32_t sdst = lds_base + (buf ^ 1) * T::kStageBytes + 2 * T::kQBytes + (wave & 1) * kStageQ * 4;
        copy4_to_lds_sv_masked((wave == 0 ? lsep : deltap) + q_src, (uint32_t)lane * 4u, sdst, wave < 2 ? copy_lanes : 0ull);
      }
    };

    // The stage is two 32-row halves (h = 0, 1).  One wave per SIMD has nobody to hide its LDS
    // and VALU latencies behind, so the four products are software-pipelined by hand:
    //   A: S, dP of half 0                    B: S, dP of half 1   | P, dS of half 0
    //   C: dV, dK with half 0 | P, dS of half 1                    D: dV, dK with half 1
    // LDS fragments are read kAhead MFMAs before their use and the scheduling fences keep the
    // written order.
    f32x16 s[2], dp[2];
    uint32_t pp[2][8], dsp[2][8];
    f32x4 lse4[2][4], dl4[2][4];
#pragma unroll
    for (int h2 = 0; h2 < 2; ++h2) {
#pragma unroll
      for (int e4 = 0; e4 < 4; ++e4) {  // element 4*e4 + x: query row 32*h2 + 8*e4 + 4g + x of the stage
        const int ql = h2 * 32 + 8 * e4 + 4 * g;
        lse4[h2][e4] = *lds_cast<const f32x4>(st + ql * 4) * kLog2e;
        dl4[h2][e4] = *lds_cast<const f32x4>(st + (kStageQ + ql) * 4);
      }
    }
    // P and dS of elements 2*pair, 2*pair + 1 of half h2 (key = this lane's, queries as above)
    auto softmax_pair = [&](int h2, int pair) {
      const int e = 2 * pair;
      const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[h2][e], c, -lse4[h2][e >> 2][e & 3]));
      const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[h2][e + 1], c, -lse4[h2][e >> 2][(e & 3) + 1]));
      pp[h2][pair] = pack_bf16(p0, p1);
      dsp[h2][pair] = pack_bf16(p0 * (dp[h2][e] - dl4[h2][e >> 2][e & 3]), p1 * (dp[h2][e + 1] - dl4[h2][e >> 2][(e & 3) + 1]));
      // keeps this arithmetic where it is written (between two MFMAs) instead of next to its first use
      asm volatile("" : "+v"(pp[h2][pair]), "+v"(dsp[h2][pair]));
    };
    // Rows that do not exist (ragged end) or that the token rule hides get P = exp(-inf) = 0 and
    // dS = 0.  Bit 16*h2 + e of `hidden` marks element e of half h2 for this lane.
    auto hide = [&](int h2) {
      if (any_hidden) {
#pragma unroll
        for (int e = 0; e < 16; ++e)
          if ((hidden >> (16 * h2 + e)) & 1u) s[h2][e] = -INFINITY;
      }
    };
    constexpr int kAhead = 2;  // in units of one k-step (two fragments) or of one transposed fragment pair
    bf16x8 qfr[2 * T::kSteps], gfr[2 * T::kSteps];
    auto read_qg = [&](int i) {  // i = h2 * kSteps + t
      const int h2 = i / T::kSteps, t = i % T::kSteps;
      qfr[i] = *lds_cast<const bf16x8>(sq + QT::piece(h2 * 32 + lq, 2 * t + g));
      gfr[i] = *lds_cast<const bf16x8>(sg + QT::piece(h2 * 32 + lq, 2 * t + g));
    };
#pragma unroll
    for (int i = 0; i < kAhead; ++i) read_qg(i);
    __builtin_amdgcn_sched_barrier(0);
    // ---- A: S, dP of half 0
#pragma unroll
    for (int t = 0; t < T::kSteps; ++t) {
      read_qg(t + kAhead);  // runs into half 1
      if (t == 0) {
        mfma32_vgpr_first(s[0], qfr[t], kf[t]);
        mfma32_vgpr_first(dp[0], gfr[t], vf[t]);
      } else {
        mfma32_vgpr(s[0], qfr[t], kf[t]);
        mfma32_vgpr(dp[0], gfr[t], vf[t]);
      }
      constexpr int kCopies = 2 * T::kQLoadsPerWave + 1;
#pragma unroll
      for (int j = t * kCopies / T::kSteps; j < (t + 1) * kCopies / T::kSteps; ++j) spread_copy(j);
      __builtin_amdgcn_sched_barrier(0);
    }
    mfma_results_settle(s[0], dp[0]);
    hide(0);
    __builtin_amdgcn_sched_barrier(0);
    // ---- B: S, dP of half 1 | P, dS of half 0
#pragma unroll
    for (int t = 0; t < T::kSteps; ++t) {
      if (t + kAhead < T::kSteps) read_qg(T::kSteps + t + kAhead);
      if (t == 0) {
        mfma32_vgpr_first(s[1], qfr[T::kSteps + t], kf[t]);
        mfma32_vgpr_first(dp[1], gfr[T::kSteps + t], vf[t]);
      } else {
        mfma32_vgpr(s[1], qfr[T::kSteps + t], kf[t]);
        mfma32_vgpr(dp[1], gfr[T::kSteps + t], vf[t]);
      }
      if (t * 8 / T::kSteps != (t + 1) * 8 / T::kSteps) softmax_pair(0, t * 8 / T::kSteps);
      if (T::kSteps == 4) softmax_pair(0, 2 * t + 1);
      __builtin_amdgcn_sched_barrier(0);
    }
    mfma_results_settle(s[1], dp[1]);
    hide(1);
    // dV^T[d, key] += dO^T[d, q] P[q, key];  dK^T[d, key] += Q^T[d, q] dS[q, key]:
    // fragment pair j = ((h2 * 2 + t2) * kDTiles + dt): transposed reads of dO and Q
    constexpr int kPairs = 2 * 2 * T::kDTiles;
    u32x4 gtr[kPairs], qtr[kPairs];
    auto read_tr = [&](int j) {
      const int h2 = j / (2 * T::kDTiles), t2 = (j / T::kDTiles) % 2, dt = j % T::kDTiles;
      const int r0 = h2 * 32 + 16 * t2 + 4 * g + (i16 >> 2);  // stage row of the first 4-row patch
      const int col = 32 * dt + 16 * half16 + 4 * (i16 & 3);
      const u32x2 g0 = lds_read_tr(sg + QT::elem(r0, col)), g1 = lds_read_tr(sg + QT::elem(r0 + 8, col));
      const u32x2 q0v = lds_read_tr(sq + QT::elem(r0, col)), q1v = lds_read_tr(sq + QT::elem(r0 + 8, col));
      gtr[j] = u32x4{g0[0], g0[1], g1[0], g1[1]};
      qtr[j] = u32x4{q0v[0], q0v[1], q1v[0], q1v[1]};
    };
#pragma unroll
    for (int j = 0; j < kAhead; ++j) read_tr(j);
    __builtin_amdgcn_sched_barrier(0);
    // ---- C: dV, dK with half 0 | P, dS of half 1;   D: dV, dK with half 1
#pragma unroll
    for (int j = 0; j < kPairs; ++j) {
      if (j + kAhead < kPairs) read_tr(j + kAhead);
      const int h2 = j / (2 * T::kDTiles), t2 = (j / T::kDTiles) % 2, dt = j % T::kDTiles;
      const bf16x8 pf = as_bf16x8(pp[h2][4 * t2], pp[h2][4 * t2 + 1], pp[h2][4 * t2 + 2], pp[h2][4 * t2 + 3]);
      const bf16x8 dsf = as_bf16x8(dsp[h2][4 * t2], dsp[h2][4 * t2 + 1], dsp[h2][4 * t2 + 2], dsp[h2][4 * t2 + 3]);
      dv[dt] = mfma32(__builtin_bit_cast(bf16x8, gtr[j]), pf, dv[dt]);
      dk[dt] = mfma32(__builtin_bit_cast(bf16x8, qtr[j]), dsf, dk[dt]);
      if (h2 == 0) {  // the 8 softmax pairs of half 1 spread over the 2 * kDTiles steps of half 0
        const int n0 = j * 8 / (2 * T::kDTiles), n1 = (j + 1) * 8 / (2 * T::kDTiles);
#pragma unroll
        for (int pair = n0; pair < n1; ++pair) softmax_pair(1, pair);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    q0 = q0_next;
    q_at = q_at_next;
  }

  // ---- epilogue: dK = scale * dK^T, dV -----------------------------------------------------
  if (key_ok) {
    __bf16* dkd = (__bf16*)a.dk.ptr + (int64_t)b * a.dk.sb + (int64_t)h * a.dk.sh + (int64_t)key_row * a.dk.sn;
    __bf16* dvd = (__bf16*)a.dv.ptr + (int64_t)b * a.dv.sb + (int64_t)h * a.dv.sh + (int64_t)key_row * a.dv.sn;
#pragma unroll
    for (int dt = 0; dt < T::kDTiles; ++dt)
#pragma unroll
      for (int e4 = 0; e4 < 4; ++e4) {
        const int d0 = 32 * dt + 8 * e4 + 4 * g;
        *(u32x2*)(dkd + d0) = u32x2{pack_bf16(dk[dt][4 * e4] * a.scale, dk[dt][4 * e4 + 1] * a.scale),
                                    pack_bf16(dk[dt][4 * e4 + 2] * a.scale, dk[dt][4 * e4 + 3] * a.scale)};
        *(u32x2*)(dvd + d0) = u32x2{pack_bf16(dv[dt][4 * e4], dv[dt][4 * e4 + 1]),
                                    pack_bf16(dv[dt][4 * e4 + 2], dv[dt][4 * e4 + 3])};
      }
  }
}

template <int D, int BLK>
struct DqTile {
  // Keys per stage of the dQ kernel.  Head dimension 128 with 64-token blocks walks half-size stages:
  // two 64-key stage buffers (64 KiB) per 2-wave workgroup would leave a compute unit with 4 waves.
  static constexpr int kStageKeys = (D == 128 && BLK == 64) ? 32 : 64;
  static constexpr int kWaves = BLK / 32;  // one wave per 32 query rows
  static constexpr int kThreads = 64 * kWaves;
  static constexpr int kSubs = BLK / kStageKeys;
  static constexpr int kSteps = D / 16;
  static constexpr int kDTiles = D / 32;
  static constexpr int kTileBytes = kStageKeys * D * 2;  // one K (or V) stage tile
  static constexpr int kLoadsPerWave = kTileBytes / 1024 / kWaves;
};

template <int D, int BLK, bool kExact>
__global__ void __launch_bounds__(2 * BLK, 2) radial_bwd_dq_kernel(const BwdArgs a) {
  using T = DqTile<D, BLK>;
  using SW = SwzTile<D>;
  // [stage buffer][K, V][kStageKeys x D bf16]
  __shared__ __attribute__((aligned(1024))) char lds[4 * T::kTileBytes];
  const uint32_t lds_base = lds_address(lds);

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lq = lane & 31;
  const int g = lane >> 5;
  const int i16 = lane & 15;
  const int half16 = (lane >> 4) & 1;

  // work item: XCD x owns the query blocks [slice[x], slice[x+1]) of every (batch, head)
  const int32_t xcd = blockIdx.x & 7;
  const int32_t s0 = a.slice[xcd];
  const int32_t slice_len = a.slice[xcd + 1] - s0;
  const int64_t idx = blockIdx.x >> 3;
  if (slice_len <= 0 || idx >= (int64_t)slice_len * a.B * a.H) return;
  const int32_t bh = (int32_t)(idx / slice_len);
  const int32_t qb = s0 + (int32_t)(idx % slice_len);
  const int32_t b = bh / a.H, h = bh % a.H;

  const __bf16* qp = (const __bf16*)a.q.ptr + (int64_t)b * a.q.sb + (int64_t)h * a.q.sh;
  const __bf16* kp = (const __bf16*)a.k.ptr + (int64_t)b * a.k.sb + (int64_t)h * a.k.sh;
  const __bf16* vp = (const __bf16*)a.v.ptr + (int64_t)b * a.v.sb + (int64_t)h * a.v.sh;
  const __bf16* gp = (const __bf16*)a.dout.ptr + (int64_t)b * a.dout.sb + (int64_t)h * a.dout.sh;

  const int32_t list_lo = __builtin_amdgcn_readfirstlane(a.row_ptr[qb]);
  const int32_t n_list = __builtin_amdgcn_readfirstlane(a.row_ptr[qb + 1]) - list_lo;
  const int32_t n_stage = n_list * T::kSubs;
  const int32_t q_row = qb * BLK + wave * 32 + lq;
  const bool q_ok = q_row < a.N;
  const int64_t q_clamped = q_ok ? q_row : a.N - 1;

  // Q and dO rows of this lane's query: B operands of S^T = K Q^T and dP^T = V dO^T.
  bf16x8 qf[T::kSteps], gf[T::kSteps];
  {
    const __bf16* qs = qp + q_clamped * a.q.sn + 8 * g;
    const __bf16* gs = gp + q_clamped * a.dout.sn + 8 * g;
#pragma unroll
    for (int t = 0; t < T::kSteps; ++t) {
      qf[t] = __builtin_bit_cast(bf16x8, *(const u32x4*)(qs + 16 * t));
      gf[t] = __builtin_bit_cast(bf16x8, *(const u32x4*)(gs + 16 * t));
    }
  }
  const float lse2 = a.lse[(int64_t)bh * a.N + q_clamped] * kLog2e;  // rows past N: values unused
  const float dlt = a.delta[(int64_t)bh * a.N + q_clamped];

  const int32_t* cols = a.col_idx + list_lo;
  int32_t cvec = lane < n_list ? cols[lane] : 0;
  int32_t nvec = 64 + lane < n_list ? cols[64 + lane] : 0;
  // token rule: (frame, position) of this lane's query and of every listed key block's first key
  StagePos q_at = {0, 0}, cvec_at = {0, 0};
  if (kExact) {
    q_at = block_pos((int32_t)q_clamped, a.rule.s);
    cvec_at = block_pos(cvec * BLK, a.rule.s);
  }

  uint32_t koff[T::kLoadsPerWave], voff[T::kLoadsPerWave];
#pragma unroll
  for (int i = 0; i < T::kLoadsPerWave; ++i) {
    int r, col;
    SW::source_of((wave * T::kLoadsPerWave + i) * 64 + lane, r, col);
    koff[i] = (uint32_t)(r * (int32_t)a.k.sn + col) * 2u;
    voff[i] = (uint32_t)(r * (int32_t)a.v.sn + col) * 2u;
  }
  // Copies the 64 K rows and V rows starting at key `key0` into stage buffer `buf`; rows past
  // N-1 are clamped to N-1 (their P is forced to zero).
  auto issue_stage = [&](int32_t key0, int buf) {
    const uint32_t kdst = lds_base + buf * 2 * T::kTileBytes + wave * T::kLoadsPerWave * 1024;
    const uint32_t vdst = kdst + T::kTileBytes;
    if (key0 + T::kStageKeys <= a.N) {
      const __bf16* kbase = kp + (int64_t)key0 * a.k.sn;  // wave-uniform
      const __bf16* vbase = vp + (int64_t)key0 * a.v.sn;
#pragma unroll
      for (int i = 0; i < T::kLoadsPerWave; ++i) copy16_to_lds_sv(kbase, koff[i], kdst + i * 1024);
#pragma unroll
      for (int i = 0; i < T::kLoadsPerWave; ++i) copy16_to_lds_sv(vbase, voff[i], vdst + i * 1024);
    } else {
      const int32_t last = a.N - 1 - key0;  // a stage wholly past N reads row N-1 only
#pragma unroll
      for (int i = 0; i < T::kLoadsPerWave; ++i) {
        int r, col;
        SW::source_of((wave * T::kLoadsPerWave + i) * 64 + lane, r, col);
        r = r < last ? r : last;
        copy16_to_lds(kp + ((int64_t)key0 + r) * a.k.sn + col, kdst + i * 1024);
        copy16_to_lds(vp + ((int64_t)key0 + r) * a.v.sn + col, vdst + i * 1024);
      }
    }
  };

  f32x16 dq[T::kDTiles];  // dQ^T: column = this lane's query, rows = d
#pragma unroll
  for (int i = 0; i < T::kDTiles; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) dq[i][e] = 0.f;
  const float c = a.scale * kLog2e;

  int32_t key0 = 0;
  StagePos k_at = {0, 0}, k_at_next = {0, 0};
  if (n_stage > 0) {
    key0 = __builtin_amdgcn_readlane(cvec, 0) * BLK;
    if (kExact) k_at = stage_pos(cvec_at, 0, 0, a.rule.s);
    issue_stage(key0, 0);
  }
  for (int32_t u = 0; u < n_stage; ++u) {
    const int buf = u & 1;
    int32_t key0_next = 0;
    const bool has_next = u + 1 < n_stage;
    if (has_next) {
      const int32_t e1 = (u + 1) / T::kSubs;
      if ((u + 1) % T::kSubs == 0 && (e1 & 63) == 0) {
        cvec = nvec;
        nvec = e1 + 64 + lane < n_list ? cols[e1 + 64 + lane] : 0;
        if (kExact) cvec_at = block_pos(cvec * BLK, a.rule.s);
      }
      key0_next = __builtin_amdgcn_readlane(cvec, e1 & 63) * BLK + ((u + 1) % T::kSubs) * T::kStageKeys;
      if (kExact) k_at_next = stage_pos(cvec_at, e1 & 63, ((u + 1) % T::kSubs) * T::kStageKeys, a.rule.s);
    }
    wait_all_copies();
    __syncthreads();

    const char* lds_k = lds + buf * 2 * T::kTileBytes;
    const char* lds_v = lds_k + T::kTileBytes;
    const bool ragged = key0 + T::kStageKeys > a.N;
    StageRule vis = {};
    bool skip = false;
    if (kExact) {
      vis = stage_rule<T::kStageKeys>(a.rule, q_at, k_at, true);  // which of the stage's keys this lane's query sees
      skip = vis.none;                             // no pair of this wave's queries with the stage's keys
    }
    // The copies of a full next stage are spread over the MFMAs of the first key tile (a burst
    // would hold the wave at the memory pipeline); a ragged next stage, or a stage this wave
    // skips, issues them at once.
    uint32_t hidden = 0u;  // bit 16kt + e: element e of key tile kt is past N or hidden by the token rule
    if (ragged || (kExact && vis.partial)) {
      uint64_t seen = stage_prefix(a.N - key0);
      if (kExact) seen &= vis.visible_mask();
      hidden = ~lane_element_bits(seen, g);
    }
    const bool any_hidden = __builtin_amdgcn_ballot_w64(hidden != 0u) != 0;
    const bool spread = has_next && !skip && key0_next + T::kStageKeys <= a.N;
    if (has_next && !spread) issue_stage(key0_next, buf ^ 1);
    if (skip) {
      key0 = key0_next;
      k_at = k_at_next;
      continue;
    }
    const uint32_t on = __builtin_amdgcn_readfirstlane(spread ? ~0u : 0u);
    const uint64_t copy_lanes = ((uint64_t)on << 32) | on;
    const int32_t key_src = spread ? key0_next : key0;  // any valid rows when the copies are switched off
    const __bf16* kbase_next = kp + (int64_t)key_src * a.k.sn;
    const __bf16* vbase_next = vp + (int64_t)key_src * a.v.sn;
    const uint32_t kdst_next = lds_base + (buf ^ 1) * 2 * T::kTileBytes + wave * T::kLoadsPerWave * 1024;
    const uint32_t vdst_next = kdst_next + T::kTileBytes;
#pragma unroll
    for (int kt = 0; kt < T::kStageKeys / 32; ++kt) {
      // S^T[key, q] and dP^T[key, q] for 32 keys x this wave's 32 queries
      f32x16 s, dp;
#pragma unroll
      for (int e = 0; e < 16; ++e) s[e] = dp[e] = 0.f;
#pragma unroll
      for (int t = 0; t < T::kSteps; ++t) {
        const bf16x8 kfrag = *lds_cast<const bf16x8>(lds_k + SW::piece(kt * 32 + lq, 2 * t + g));
        const bf16x8 vfrag = *lds_cast<const bf16x8>(lds_v + SW::piece(kt * 32 + lq, 2 * t + g));
        s = mfma32(kfrag, qf[t], s);
        dp = mfma32(vfrag, gf[t], dp);
        if (kt == 0) {  // 2 * kLoadsPerWave copies over the kSteps steps of the first key tile
          constexpr int kCopies = 2 * T::kLoadsPerWave;
#pragma unroll
          for (int j = t * kCopies / T::kSteps; j < (t + 1) * kCopies / T::kSteps; ++j) {
            if (j < T::kLoadsPerWave) copy16_to_lds_sv_masked(kbase_next, koff[j], kdst_next + j * 1024, copy_lanes);
            else copy16_to_lds_sv_masked(vbase_next, voff[j - T::kLoadsPerWave], vdst_next + (j - T::kLoadsPerWave) * 1024, copy_lanes);
          }
        }
      }
      // element e: key = key0 + 32kt + 8(e/4) + 4g + e%4, query = q_row (this lane)
      if (any_hidden) {  // hidden pairs: P = exp(-inf) = 0
#pragma unroll
        for (int e = 0; e < 16; ++e)
          if ((hidden >> (16 * kt + e)) & 1u) s[e] = -INFINITY;
      }
      uint32_t dsp[8];
#pragma unroll
      for (int e = 0; e < 16; e += 2) {
        const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[e], c, -lse2));
        const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[e + 1], c, -lse2));
        dsp[e >> 1] = pack_bf16(p0 * (dp[e] - dlt), p1 * (dp[e + 1] - dlt));
      }
      // dQ^T[d, q] += K^T[d, key] dS^T[key, q]
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2) {
        const bf16x8 dsf = as_bf16x8(dsp[4 * t2], dsp[4 * t2 + 1], dsp[4 * t2 + 2], dsp[4 * t2 + 3]);
        const int r0 = kt * 32 + 16 * t2 + 4 * g + (i16 >> 2);
#pragma unroll
        for (int dt = 0; dt < T::kDTiles; ++dt) {
          const int col = 32 * dt + 16 * half16 + 4 * (i16 & 3);
          const u32x2 k0 = lds_read_tr(lds_k + SW::elem(r0, col)), k1 = lds_read_tr(lds_k + SW::elem(r0 + 8, col));
          dq[dt] = mfma32(as_bf16x8(k0[0], k0[1], k1[0], k1[1]), dsf, dq[dt]);
        }
      }
    }
    key0 = key0_next;
    k_at = k_at_next;
  }

  if (q_ok) {
    __bf16* dst = (__bf16*)a.dq.ptr + (int64_t)b * a.dq.sb + (int64_t)h * a.dq.sh + (int64_t)q_row * a.dq.sn;
#pragma unroll
    for (int dt = 0; dt < T::kDTiles; ++dt)
#pragma unroll
      for (int e4 = 0; e4 < 4; ++e4)  // dq[dt][4*e4 + x] is d = 32dt + 8*e4 + 4g + x
        *(u32x2*)(dst + 32 * dt + 8 * e4 + 4 * g) =
            u32x2{pack_bf16(dq[dt][4 * e4] * a.scale, dq[dt][4 * e4 + 1] * a.scale),
                  pack_bf16(dq[dt][4 * e4 + 2] * a.scale, dq[dt][4 * e4 + 3] * a.scale)};
  }
}

template <int D, int BLK, bool kExact>
int launch(const BwdArgs& a, hipStream_t stream) {
  using T = BwdTile<D, BLK>;
  const int64_t rows = (int64_t)a.B * a.H * a.N;
  const int rows_per_block = 256 / (D / 8);
  const int64_t prep_grid = (rows + rows_per_block - 1) / rows_per_block;
  const int64_t grid_kv = 8LL * a.B * a.H * a.max_slice_t;
  const int64_t grid_q = 8LL * a.B * a.H * a.max_slice;
  if (prep_grid > 0x7fffffffLL || grid_kv > 0x7fffffffLL || grid_q > 0x7fffffffLL)
    return fail(RADIAL_ESHAPE, "problem too large for one launch");
  // The dK/dV kernel needs more dynamic LDS than the default limit.  The attribute belongs to the
  // (device, kernel) pair; it is set once per device and template instance.  Setting it twice is
  // harmless, so two host threads racing through here only repeat the call.
  static std::atomic<bool> configured[kMaxDevices];
  int dev = 0;
  RADIAL_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices || !configured[dev].load(std::memory_order_acquire)) {
    RADIAL_HIP_TRY(hipFuncSetAttribute((const void*)radial_bwd_dkdv_kernel<D, BLK, kExact>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, T::kLdsBytes));
    if (dev >= 0 && dev < kMaxDevices) configured[dev].store(true, std::memory_order_release);
  }
  bwd_prepare_kernel<D><<<dim3((unsigned)prep_grid), dim3(256), 0, stream>>>(a);
  if (grid_kv > 0)
    radial_bwd_dkdv_kernel<D, BLK, kExact><<<dim3((unsigned)grid_kv), dim3(T::kThreads), T::kLdsBytes, stream>>>(a);
  if (grid_q > 0)
    radial_bwd_dq_kernel<D, BLK, kExact><<<dim3((unsigned)grid_q), dim3(DqTile<D, BLK>::kThreads), 0, stream>>>(a);
  RADIAL_HIP_TRY(hipGetLastError());
  return RADIAL_OK;
}

template <int D, int BLK>
int launch(const BwdArgs& a, hipStream_t stream) {
  return a.rule.exact ? launch<D, BLK, true>(a, stream) : launch<D, BLK, false>(a, stream);
}

}  // namespace

int launch_bwd(int D, int block, const BwdArgs& a, hipStream_t stream) {
  if (D == 128 && block == 128) return launch<128, 128>(a, stream);
  if (D == 64 && block == 128) return launch<64, 128>(a, stream);
  if (D == 128 && block == 64) return launch<128, 64>(a, stream);
  if (D == 64 && block == 64) return launch<64, 64>(a, stream);
  return fail(RADIAL_EUNSUPPORTED, "head dimension %d with block %d is not supported", D, block);
}

}  // namespace radial
