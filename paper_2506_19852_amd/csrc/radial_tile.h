// Device helpers shared by the attention kernels: MFMA operand types, LDS tile addressing,
// HBM -> LDS copies.  gfx950 only.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "radial_internal.h"

namespace radial {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

// Generic pointer into a __shared__ array -> LDS (address space 3) pointer.
template <class T>
__device__ __forceinline__ __attribute__((address_space(3))) T* lds_cast(const void* p) {
  return (__attribute__((address_space(3))) T*)(p);
}

__device__ __forceinline__ uint32_t lds_address(const void* p) { return (uint32_t)(uintptr_t)lds_cast<char>(p); }

// v_mfma_f32_32x32x16_bf16: D[32x32] += A[32x16] * B[16x32].
//   A: lane l holds row l%32, k = 8*(l/32) .. +7;   B: lane l holds column l%32, same k;
//   D: lane l holds column l%32, element e is row 8*(e/4) + 4*(l/32) + e%4.
// A and B have the same register layout, so swapping them transposes the product.
__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  f32x2 f = {a, b};
  bf16x2 h = __builtin_convertvector(f, bf16x2);
  return __builtin_bit_cast(uint32_t, h);
}

__device__ __forceinline__ bf16x8 as_bf16x8(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
  const u32x4 raw = {a, b, c, d};
  return __builtin_bit_cast(bf16x8, raw);
}

// One 1 KiB HBM -> LDS copy: lane i's 16 bytes land at LDS address lds_addr + 16*i.  Issued
// from assembly so that the compiler does not order later LDS reads after it; the caller
// waits with wait_all_copies() and a barrier before anyone reads the destination.
__device__ __forceinline__ void copy16_to_lds(const void* gptr, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(gptr) : "memory", "m0");
}
// copy16_to_lds with the address split into a wave-uniform 64-bit base (SGPRs) and a per-lane
// 32-bit byte offset, so that walking to the next tile costs scalar arithmetic only.
__device__ __forceinline__ void copy16_to_lds_sv(const void* base, uint32_t byte_offset, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr), "v"(byte_offset), "s"(base) : "memory", "m0");
}
// copy16_to_lds_sv for the lanes set in `lanes` only (all or none in practice: with no lane the
// instruction is a no-op, which lets straight-line code switch a copy off without a branch).
__device__ __forceinline__ void copy16_to_lds_sv_masked(const void* base, uint32_t byte_offset, uint32_t lds_addr, uint64_t lanes) {
  // `lanes` is wave-uniform by contract; say so to the compiler (the operand must be scalar)
  lanes = ((uint64_t)__builtin_amdgcn_readfirstlane((uint32_t)(lanes >> 32)) << 32) | __builtin_amdgcn_readfirstlane((uint32_t)lanes);
  uint64_t saved;
  asm volatile("s_mov_b32 m0, %1\n\ts_and_saveexec_b64 %0, %4\n\tglobal_load_lds_dwordx4 %2, %3\n\ts_mov_b64 exec, %0"
               : "=&s"(saved) : "s"(lds_addr), "v"(byte_offset), "s"(base), "s"(lanes) : "memory", "scc", "m0");
}
// The 4-byte form of copy16_to_lds_sv_masked (256 bytes per wave).
__device__ __forceinline__ void copy4_to_lds_sv_masked(const void* base, uint32_t byte_offset, uint32_t lds_addr, uint64_t lanes) {
  // `lanes` is wave-uniform by contract; say so to the compiler (the operand must be scalar)
  lanes = ((uint64_t)__builtin_amdgcn_readfirstlane((uint32_t)(lanes >> 32)) << 32) | __builtin_amdgcn_readfirstlane((uint32_t)lanes);
  uint64_t saved;
  asm volatile("s_mov_b32 m0, %1\n\ts_and_saveexec_b64 %0, %4\n\tglobal_load_lds_dword %2, %3\n\ts_mov_b64 exec, %0"
               : "=&s"(saved) : "s"(lds_addr), "v"(byte_offset), "s"(base), "s"(lanes) : "memory", "scc", "m0");
}
// Same as copy16_to_lds with 4 bytes per lane (256 bytes per wave).
__device__ __forceinline__ void copy4_to_lds(const void* gptr, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off" ::"s"(lds_addr), "v"(gptr) : "memory", "m0");
}
__device__ __forceinline__ void wait_all_copies() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// A [rows x kRowElems] bf16 tile in LDS, cut into 16-byte pieces and 256-byte lines.  Pieces
// are XOR-swizzled inside their line so that both access patterns used on a tile are free of
// bank conflicts: 128-bit reads of one piece column over 16 consecutive rows, and the 64-bit
// transposing reads (ds_read_b64_tr_b16) that touch 4 consecutive rows x 64 bytes.
template <int kRowElems>
struct SwzTile {
  static_assert(kRowElems == 64 || kRowElems == 128, "row of 128 or 256 bytes");
  static constexpr int kPieces = kRowElems / 8;
  __device__ static __forceinline__ int key(int line) {
    return kRowElems == 128 ? (((line & 3) << 2) | ((line >> 2) & 3)) : (((line & 1) << 2) | ((line >> 1) & 3));
  }
  // byte offset of piece p of row r
  __device__ static __forceinline__ int piece(int r, int p) {
    const int lin = r * kPieces + p;
    const int line = lin >> 4, slot = lin & 15;
    return (line << 8) + ((slot ^ key(line)) << 4);
  }
  // byte offset of element (r, c); c % 4 == 0 for the 8-byte accesses
  __device__ static __forceinline__ int elem(int r, int c) { return piece(r, c >> 3) + ((c & 7) << 1); }
  // (row, first element) of the source piece that belongs at linear LDS piece index `lin`
  __device__ static __forceinline__ void source_of(int lin, int& r, int& c) {
    const int line = lin >> 4, slot = lin & 15;
    const int src = (line << 4) + (slot ^ key(line));
    r = src / kPieces;
    c = (src % kPieces) * 8;
  }
};

// Transposing LDS read: within each group of 16 lanes, lane i supplies the address of 4
// consecutive bf16 of row i/4 (columns 4*(i%4)..) and receives, for column i of that 16-wide
// patch, the values of the group's 4 rows.
__device__ __forceinline__ u32x2 lds_read_tr(const char* p) {
  const s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16(lds_cast<s16x4>(p));
  return __builtin_bit_cast(u32x2, v);
}

// max(x, value of x in lane^32), exchanged in registers (v_permlane32_swap: the upper 32 lanes
// of the first operand trade places with the lower 32 lanes of the second).
__device__ __forceinline__ float max_with_other_half(float x) {
  const uint32_t u = __builtin_bit_cast(uint32_t, x);
  const auto sw = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  // Copy the elements out before reinterpreting them: a bit_cast applied directly to
  // sw[1] reads element 0.
  const uint32_t first = sw[0], second = sw[1];
  return fmaxf(__builtin_bit_cast(float, first), __builtin_bit_cast(float, second));
}

// ---- token-level rule of the radial mask inside listed blocks ---------------------------------
// (Sec. 4.2 of the paper, formal definition, plus the attention sink of App. A.1.)

// For one (query frame i, key frame j) pair: the largest |k - l| a query position k may
// attend; -1 = nothing, >= s - 1 = the whole frame.
__device__ __forceinline__ int32_t radial_half_width(const TokenRule& rule, int32_t i, int32_t j) {
  if (j < rule.sink || i >= rule.frames || j >= rule.frames) return rule.s;  // sink, text tokens
  const int32_t d = i > j ? i - j : j - i;
  if (rule.half_width) return rule.half_width[d];  // banded pattern: table lookup (d <= frames)
  if (d < 2) return rule.s - 1;            // band 0: the whole frame, never scaled
  const int32_t r = 31 - __clz(d);         // floor(log2 d)
  const int32_t w = rule.w0 >> r;          // diagonal width floor(c*s / 2^r)
  if (w >= 1) return (w < rule.s ? w : rule.s) - 1;
  const int64_t b_den = (int64_t)rule.den << r;
  const int32_t stride = (int32_t)((b_den + rule.s_num - 1) / rule.s_num);
  return d % stride == 0 ? 0 : -1;         // sub-sampled single diagonals
}

// A stage is 64 (or 32) consecutive tokens (keys for the query-stationary kernels, queries for the
// key-stationary one) that start at (frame, pos).  With s >= 64 it touches at most the two
// frames `frame` and `frame + 1`.
struct StagePos {
  int32_t frame, pos;
};

// (frame, position) of token index `block_start` for every lane's list entry.
__device__ __forceinline__ StagePos block_pos(int32_t block_start, int32_t s) {
  StagePos r;
  r.frame = block_start / s;
  r.pos = block_start - r.frame * s;
  return r;
}

// Entry `idx` of the per-lane positions, advanced by `offset` (< 128) tokens; wave-uniform.
__device__ __forceinline__ StagePos stage_pos(StagePos per_lane, int idx, int32_t offset, int32_t s) {
  StagePos r;
  r.frame = __builtin_amdgcn_readlane(per_lane.frame, idx);
  r.pos = __builtin_amdgcn_readlane(per_lane.pos, idx) + offset;
  if (r.pos >= s) {
    r.pos -= s;
    r.frame += 1;
  }
  return r;
}

// What one lane's token (its own frame/position, a query or a key) sees of a stage: tokens
// [lo0, lo0 + n0) of the stage's first frame and [lo1, lo1 + n1) of its second, as offsets
// 0..63 into the stage.
struct StageRule {
  int32_t lo0, lo1;
  uint32_t n0, n1;
  bool partial;  // wave-uniform: some lane of the wave has a hidden pair in this stage
  bool none;     // wave-uniform: no lane of the wave has a visible pair in this stage

  // token `x` (0..63) of the stage
  __device__ __forceinline__ bool visible(int x) const {
    return ((uint32_t)(x - lo0) < n0) | ((uint32_t)(x - lo1) < n1);  // n1 = 0 without a second frame
  }
  // bit x set iff token x of the stage is visible
  __device__ __forceinline__ uint64_t visible_mask() const { return stage_interval(lo0, n0) | stage_interval(lo1, n1); }
  // bits [lo, lo + n) of a 64-token stage (n = 0: none; lo + n <= 64 otherwise)
  __device__ static __forceinline__ uint64_t stage_interval(int32_t lo, uint32_t n) {
    if (n == 0u) return 0ull;
    const uint64_t ones = n >= 64u ? ~0ull : ((1ull << n) - 1ull);
    return ones << lo;
  }
};

// The first `count` tokens of a stage (count >= 64: all of them): those that exist before N.
__device__ __forceinline__ uint64_t stage_prefix(int32_t count) {
  return count >= 64 ? ~0ull : (count <= 0 ? 0ull : ((1ull << count) - 1ull));
}

// An MFMA accumulator pair (two 32-token tiles of a stage) holds, in lane group g = lane/32,
// element e of tile kt for stage token 32kt + 8(e/4) + 4g + e%4.  From a mask over the 64 stage
// tokens this returns the lane's 32 bits in element order (bit 16kt + e): nibble g of every
// byte of the mask, packed.
__device__ __forceinline__ uint32_t lane_element_bits(uint64_t token_mask, int g) {
  uint64_t v = (token_mask >> (4 * g)) & 0x0F0F0F0F0F0F0F0Full;
  v = (v | (v >> 4)) & 0x00FF00FF00FF00FFull;
  v = (v | (v >> 8)) & 0x0000FFFF0000FFFFull;
  v = (v | (v >> 16));
  return (uint32_t)v;
}

// own_is_query: the lane holds a query and the stage holds keys; otherwise the reverse.
// kWidth: tokens in the stage (64, or 32 for the kernels that walk half-size stages).
template <int kWidth = 64>
__device__ __forceinline__ StageRule stage_rule(const TokenRule& rule, StagePos own, StagePos stage, bool own_is_query) {
  const int32_t s = rule.s;
  const int32_t hw0 = own_is_query ? radial_half_width(rule, own.frame, stage.frame)
                                   : radial_half_width(rule, stage.frame, own.frame);
  const int32_t hw1 = own_is_query ? radial_half_width(rule, own.frame, stage.frame + 1)
                                   : radial_half_width(rule, stage.frame + 1, own.frame);
  const int32_t split = s - stage.pos;  // stage offset at which the second frame starts
  StageRule r;
  // first frame: positions stage.pos + x, x in [0, min(split, kWidth)), within hw0 of own.pos
  const int32_t a0 = max(own.pos - hw0 - stage.pos, 0), b0 = min(own.pos + hw0 - stage.pos, min(split, kWidth) - 1);
  r.lo0 = a0;
  r.n0 = b0 >= a0 ? (uint32_t)(b0 - a0 + 1) : 0u;
  // second frame: positions x - split, x in [split, kWidth), within hw1 of own.pos
  const int32_t a1 = max(own.pos - hw1 + split, split), b1 = min(own.pos + hw1 + split, kWidth - 1);
  r.lo1 = a1;
  r.n1 = b1 >= a1 ? (uint32_t)(b1 - a1 + 1) : 0u;
  const bool all_visible = r.n0 + r.n1 == (uint32_t)kWidth;
  r.partial = __builtin_amdgcn_ballot_w64(!all_visible) != 0;
  r.none = __builtin_amdgcn_ballot_w64(r.n0 + r.n1 != 0u) == 0;
  return r;
}

}  // namespace radial
