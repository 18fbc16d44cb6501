// Device helpers shared by the attention kernels: MFMA operand types, LDS tile addressing,
// HBM -> LDS copies.  gfx950 only.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

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
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(gptr) : "memory");
}
// copy16_to_lds with the address split into a wave-uniform 64-bit base (SGPRs) and a per-lane
// 32-bit byte offset, so that walking to the next tile costs scalar arithmetic only.
__device__ __forceinline__ void copy16_to_lds_sv(const void* base, uint32_t byte_offset, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr), "v"(byte_offset), "s"(base) : "memory");
}
// Same as copy16_to_lds with 4 bytes per lane (256 bytes per wave).
__device__ __forceinline__ void copy4_to_lds(const void* gptr, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off" ::"s"(lds_addr), "v"(gptr) : "memory");
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

}  // namespace radial
