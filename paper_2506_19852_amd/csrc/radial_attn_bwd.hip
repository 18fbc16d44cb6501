// Block-sparse attention backward for gfx950: the gradient of Eq. 2 of the paper restricted to
// the listed block pairs,
//     P = exp(scale*Q K^T - LSE),  dV = P^T dO,  dP = dO V^T,  delta = rowsum(dO * O),
//     dS = P * (dP - delta),       dQ = scale * dS K,          dK = scale * dS^T Q.
//
// Three kernels:
//   prepare : delta[b,h,q] = sum_d dO*O, and zero the fp32 dQ accumulator;
//   main    : one workgroup per (batch, head, key block) walks the transposed list (the query
//             blocks that list this key block) in stages of 64 query rows.  Wave w owns 32
//             keys; its K and V rows stay in registers, dK^T and dV^T accumulate in registers
//             (column = key = lane%32).  S and dP are computed with query rows as MFMA rows
//             so that P and dS come out with keys across lanes: 8 accumulator rows at a time
//             they are the B operands of dV^T += dO^T P and dK^T += Q^T dS, whose A operands
//             are transposing LDS reads of the dO and Q stage tiles.  dS is also parked in
//             LDS (key-major) so that, after a barrier, the waves split dQ = dS K of the stage
//             by output tile and add it to the fp32 accumulator with atomics;
//   finish  : dQ accumulator -> bf16.
// Q and dO stage tiles, LSE and delta are copied HBM -> LDS by global_load_lds, double
// buffered, one stage ahead.
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
  static constexpr int kKBytes = BLK * D * 2;            // K tile, key-major (read transposed for dQ)
  static constexpr int kQBytes = kStageQ * D * 2;        // Q or dO stage tile
  static constexpr int kStatBytes = 2 * kStageQ * 4;     // LSE and delta of a stage
  static constexpr int kStageBytes = 2 * kQBytes + kStatBytes;
  static constexpr int kDsBytes = BLK * kStageQ * 2;     // dS^T tile [key][64 q]
  static constexpr int kLdsBytes = kKBytes + 2 * kStageBytes + kDsBytes;
  static constexpr int kKLoadsPerWave = kKBytes / 1024 / kWaves;
  static constexpr int kQLoadsPerWave = kQBytes / 1024 / kWaves;
  static constexpr int kDqTilesPerWave = 2 * kDTiles / kWaves;  // 32x32 dQ tiles per wave per stage
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
    f32x4* acc = (f32x4*)(a.dq_acc + row * D + piece * 8);
    acc[0] = f32x4{0.f, 0.f, 0.f, 0.f};
    acc[1] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
#pragma unroll
  for (int off = kLanesPerRow / 2; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
  if (row < rows && piece == 0) a.delta[row] = sum;
}

template <int D>
__global__ void __launch_bounds__(256) bwd_finish_kernel(const BwdArgs a) {
  constexpr int kLanesPerRow = D / 8;
  const int64_t rows = (int64_t)a.B * a.H * a.N;
  const int64_t row = (int64_t)blockIdx.x * (256 / kLanesPerRow) + threadIdx.x / kLanesPerRow;
  const int piece = threadIdx.x % kLanesPerRow;
  if (row >= rows) return;
  const int32_t q = (int32_t)(row % a.N);
  const int32_t bh = (int32_t)(row / a.N);
  const int32_t b = bh / a.H, h = bh % a.H;
  const f32x4* acc = (const f32x4*)(a.dq_acc + row * D + piece * 8);
  const f32x4 x = acc[0], y = acc[1];
  u32x4 w = {pack_bf16(x[0], x[1]), pack_bf16(x[2], x[3]), pack_bf16(y[0], y[1]), pack_bf16(y[2], y[3])};
  __bf16* dst = (__bf16*)a.dq.ptr + (int64_t)b * a.dq.sb + (int64_t)h * a.dq.sh + (int64_t)q * a.dq.sn + piece * 8;
  *(u32x4*)dst = w;
}

template <int D, int BLK>
__global__ void __launch_bounds__(2 * BLK, 1) radial_bwd_kernel(const BwdArgs a) {
  using T = BwdTile<D, BLK>;
  using QT = SwzTile<D>;         // K, Q, dO tiles: rows of D elements
  using ST = SwzTile<kStageQ>;   // dS^T tile: rows of 64 query positions
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  char* const lds_kt = lds;
  char* const lds_ds = lds + T::kKBytes + 2 * T::kStageBytes;
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
  float* dqp = a.dq_acc + (int64_t)bh * a.N * D;

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

  // the K tile, key-major, for the transposing reads of the dQ product
#pragma unroll
  for (int i = 0; i < T::kKLoadsPerWave; ++i) {
    const int chunk = wave * T::kKLoadsPerWave + i;
    int r, c;
    QT::source_of(chunk * 64 + lane, r, c);
    int32_t row = kb * BLK + r;
    row = row < a.N ? row : a.N - 1;
    copy16_to_lds(kp + (int64_t)row * a.k.sn + c, lds_base + chunk * 1024);
  }

  const int32_t* rows_list = a.row_idx + list_lo;
  int32_t cvec = lane < n_list ? rows_list[lane] : 0;
  int32_t nvec = 64 + lane < n_list ? rows_list[64 + lane] : 0;

  int32_t srow[T::kQLoadsPerWave], scol[T::kQLoadsPerWave];
#pragma unroll
  for (int i = 0; i < T::kQLoadsPerWave; ++i) QT::source_of((wave * T::kQLoadsPerWave + i) * 64 + lane, srow[i], scol[i]);

  // Copies Q, dO (64 rows from q0) and their LSE / delta into stage buffer `buf`.
  auto issue_stage = [&](int32_t q0, int buf) {
    const uint32_t qdst = lds_base + T::kKBytes + buf * T::kStageBytes + wave * T::kQLoadsPerWave * 1024;
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
      const uint32_t sdst = lds_base + T::kKBytes + buf * T::kStageBytes + 2 * T::kQBytes + wave * kStageQ * 4;
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
  if (n_stage > 0) {
    q0 = __builtin_amdgcn_readlane(cvec, 0) * BLK;
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
      }
      q0_next = __builtin_amdgcn_readlane(cvec, e1 & 63) * BLK + ((u + 1) % T::kSubs) * kStageQ;
    }

    wait_all_copies();  // stage u (and, the first time, the K tile) has landed
    __syncthreads();    // for every wave; stage u-1 including its dQ phase is finished
    if (has_next) issue_stage(q0_next, buf ^ 1);

    const char* sq = lds + T::kKBytes + buf * T::kStageBytes;
    const char* sg = sq + T::kQBytes;
    const char* st = sg + T::kQBytes;  // 64 x LSE then 64 x delta
    const bool ragged_q = q0 + kStageQ > a.N;

#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
      // S[q, key] and dP[q, key] for 32 query rows x this wave's 32 keys
      f32x16 s, dp;
#pragma unroll
      for (int e = 0; e < 16; ++e) s[e] = dp[e] = 0.f;
#pragma unroll
      for (int t = 0; t < T::kSteps; ++t) {
        const bf16x8 qfrag = *lds_cast<const bf16x8>(sq + QT::piece(qt * 32 + lq, 2 * t + g));
        const bf16x8 gfrag = *lds_cast<const bf16x8>(sg + QT::piece(qt * 32 + lq, 2 * t + g));
        s = mfma32(qfrag, kf[t], s);
        dp = mfma32(gfrag, vf[t], dp);
      }
      // element e: key = key_row (this lane), query = q0 + 32qt + 8(e/4) + 4g + e%4
      uint32_t pp[8], dsp[8];
#pragma unroll
      for (int e4 = 0; e4 < 4; ++e4) {
        const int ql = qt * 32 + 8 * e4 + 4 * g;
        const f32x4 lse4 = *lds_cast<const f32x4>(st + ql * 4);
        const f32x4 dl4 = *lds_cast<const f32x4>(st + (kStageQ + ql) * 4);
        float p[4], ds[4];
#pragma unroll
        for (int x = 0; x < 4; ++x) {
          p[x] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[4 * e4 + x], c, -lse4[x] * kLog2e));
          if (!key_ok || (ragged_q && q0 + ql + x >= a.N)) p[x] = 0.f;
          ds[x] = p[x] * (dp[4 * e4 + x] - dl4[x]);
        }
        pp[2 * e4] = pack_bf16(p[0], p[1]);
        pp[2 * e4 + 1] = pack_bf16(p[2], p[3]);
        dsp[2 * e4] = pack_bf16(ds[0], ds[1]);
        dsp[2 * e4 + 1] = pack_bf16(ds[2], ds[3]);
        // park dS^T[key][q]: 4 consecutive query positions
        *lds_cast<u32x2>(lds_ds + ST::elem(wave * 32 + lq, ql)) = u32x2{dsp[2 * e4], dsp[2 * e4 + 1]};
      }
      // dV^T[d, key] += dO^T[d, q] P[q, key];  dK^T[d, key] += Q^T[d, q] dS[q, key]
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2) {
        const bf16x8 pf = as_bf16x8(pp[4 * t2], pp[4 * t2 + 1], pp[4 * t2 + 2], pp[4 * t2 + 3]);
        const bf16x8 dsf = as_bf16x8(dsp[4 * t2], dsp[4 * t2 + 1], dsp[4 * t2 + 2], dsp[4 * t2 + 3]);
        const int r0 = qt * 32 + 16 * t2 + 4 * g + (i16 >> 2);  // stage row of the first 4-row patch
#pragma unroll
        for (int dt = 0; dt < T::kDTiles; ++dt) {
          const int col = 32 * dt + 16 * half16 + 4 * (i16 & 3);
          const u32x2 g0 = lds_read_tr(sg + QT::elem(r0, col)), g1 = lds_read_tr(sg + QT::elem(r0 + 8, col));
          dv[dt] = mfma32(as_bf16x8(g0[0], g0[1], g1[0], g1[1]), pf, dv[dt]);
          const u32x2 q0v = lds_read_tr(sq + QT::elem(r0, col)), q1v = lds_read_tr(sq + QT::elem(r0 + 8, col));
          dk[dt] = mfma32(as_bf16x8(q0v[0], q0v[1], q1v[0], q1v[1]), dsf, dk[dt]);
        }
      }
    }
    __syncthreads();  // dS^T of all keys of the block is in LDS

    // dQ[q, d] += scale * dS[q, :] K[:, d]: this wave's share of the 2 x kDTiles output tiles
#pragma unroll
    for (int j = 0; j < T::kDqTilesPerWave; ++j) {
      const int ti = wave * T::kDqTilesPerWave + j;
      const int qt = ti / T::kDTiles, dt = ti % T::kDTiles;
      f32x16 acc;
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[e] = 0.f;
#pragma unroll
      for (int t3 = 0; t3 < BLK / 16; ++t3) {
        const int kr = 16 * t3 + 4 * g + (i16 >> 2);  // key row of the first 4-key patch
        const int qc = qt * 32 + 16 * half16 + 4 * (i16 & 3);
        const int dc = 32 * dt + 16 * half16 + 4 * (i16 & 3);
        const u32x2 a0 = lds_read_tr(lds_ds + ST::elem(kr, qc)), a1 = lds_read_tr(lds_ds + ST::elem(kr + 8, qc));
        const u32x2 b0 = lds_read_tr(lds_kt + QT::elem(kr, dc)), b1 = lds_read_tr(lds_kt + QT::elem(kr + 8, dc));
        acc = mfma32(as_bf16x8(a0[0], a0[1], a1[0], a1[1]), as_bf16x8(b0[0], b0[1], b1[0], b1[1]), acc);
      }
      // acc element e: query q0 + 32qt + 8(e/4) + 4g + e%4, column d = 32dt + lq
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int32_t q = q0 + qt * 32 + 8 * (e >> 2) + 4 * g + (e & 3);
        if (q < a.N) unsafeAtomicAdd(dqp + (int64_t)q * D + 32 * dt + lq, acc[e] * a.scale);
      }
    }
    q0 = q0_next;
  }

  // ---- epilogue: dK = scale * dK^T, dV -----------------------------------------------------
  if (n_stage == 0) wait_all_copies();  // nothing may stay in flight when the wave ends
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
int launch(const BwdArgs& a, hipStream_t stream) {
  using T = BwdTile<D, BLK>;
  const int64_t rows = (int64_t)a.B * a.H * a.N;
  const int rows_per_block = 256 / (D / 8);
  const int64_t prep_grid = (rows + rows_per_block - 1) / rows_per_block;
  const int64_t grid = 8LL * a.B * a.H * a.max_slice_t;
  if (prep_grid > 0x7fffffffLL || grid > 0x7fffffffLL) return fail(RADIAL_ESHAPE, "problem too large for one launch");
  static bool configured = false;  // per template instance
  if (!configured) {
    RADIAL_HIP_TRY(hipFuncSetAttribute((const void*)radial_bwd_kernel<D, BLK>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       T::kLdsBytes));
    configured = true;
  }
  bwd_prepare_kernel<D><<<dim3((unsigned)prep_grid), dim3(256), 0, stream>>>(a);
  if (grid > 0) radial_bwd_kernel<D, BLK><<<dim3((unsigned)grid), dim3(T::kThreads), T::kLdsBytes, stream>>>(a);
  bwd_finish_kernel<D><<<dim3((unsigned)prep_grid), dim3(256), 0, stream>>>(a);
  RADIAL_HIP_TRY(hipGetLastError());
  return RADIAL_OK;
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
