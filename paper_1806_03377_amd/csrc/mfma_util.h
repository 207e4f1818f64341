// MFMA fragment types and LDS tile helpers shared by the bf16 GEMM and convolution kernels (gfx950).
//
// Operand layout of v_mfma_f32_32x32x16_bf16 as used here (wave = 64 lanes, lane l):
//   A fragment: row (l & 31) of a 32 x 16 block, reduction elements 8*(l >> 5) .. +7   (16 bytes)
//   B fragment: column (l & 31) of a 16 x 32 block, same reduction elements           (16 bytes)
//   D (16 floats): column (l & 31), rows 8*(r / 4) + 4*(l >> 5) + (r % 4) for r = 0..15
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pd_kernels.h"

namespace pd {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ bf16x8 frag(uint4 v) { return __builtin_bit_cast(bf16x8, v); }


constexpr int kThreads = 256;

__device__ __forceinline__ uint4 ldg16(const bf16_t* p) { return *reinterpret_cast<const uint4*>(p); }
__device__ __forceinline__ uint4 zero16() { return make_uint4(0u, 0u, 0u, 0u); }
// 16-byte load of data that is read once per kernel (a weight stream): non-temporal, so that it does not push
// reusable lines (activations, partial sums) out of the caches
typedef unsigned int vu4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 ldg16_stream(const bf16_t* p) {
  const vu4_t v = __builtin_nontemporal_load(reinterpret_cast<const vu4_t*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}

// One wave-wide 16-byte-per-lane load straight from global memory into LDS (global_load_lds_dwordx4): lane L's
// chunk, read from `uniform_base` + `lane_byte_offset`, lands at `uniform_lds_dst` + 16 L.  Written as inline
// assembly: for the builtin the compiler inserts a wait for ALL outstanding loads before every LDS read, which
// serialises a pipeline; the caller waits with an explicit s_waitcnt vmcnt(n) instead.
typedef __attribute__((address_space(3))) void lds_void_t;
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void dma_load16(const bf16_t* uniform_base, uint32_t lane_byte_offset, char* uniform_lds_dst) {
  const uint32_t lds_addr =
      __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_void_t*)(uniform_lds_dst));
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(lane_byte_offset), "s"(uniform_base), "s"(lds_addr)
               : "memory", "m0");
}
// The same with the LDS destination given as a 32-bit LDS address that the caller has formed once (lds_address_of
// below) plus uniform arithmetic of its own: converting a generic pointer per load costs a null check and a select
// (four scalar instructions in front of every load, a dependent chain in a wave whose time belongs to the MFMAs).
__device__ __forceinline__ uint32_t lds_address_of(const void* p) {
  return __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_void_t*)(p));
}
__device__ __forceinline__ void dma_load16_at(const bf16_t* uniform_base, uint32_t lane_byte_offset, uint32_t uniform_lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(lane_byte_offset), "s"(uniform_base), "s"(uniform_lds_addr)
               : "memory", "m0");
}
// the same for data that is read once per kernel (a weight stream): non-temporal, so that it is not kept in the
// caches at the expense of reusable lines
__device__ __forceinline__ void dma_load16_stream(const bf16_t* uniform_base, uint32_t lane_byte_offset,
                                                  char* uniform_lds_dst) {
  const uint32_t lds_addr =
      __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_void_t*)(uniform_lds_dst));
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt"
               :
               : "v"(lane_byte_offset), "s"(uniform_base), "s"(lds_addr)
               : "memory", "m0");
}
#pragma clang diagnostic pop

// XOR swizzle of the 16-byte groups of an LDS row that holds 8*G reduction elements of one output row/column
// (G groups).  Spreads both the transposing 4-byte writes (lanes differ in their column chunk and reduction
// pair) and the 16-byte fragment reads (lanes differ in their row) over all banks.
template <int G>
__device__ __forceinline__ int swz(int row, int group) {
  return group ^ ((row ^ (row >> 3)) & ((G < 16 ? G : 16) - 1));
}

// Writes an 8-column x 2-row block (two 16-byte global chunks from consecutive reduction rows `pair`*2,
// `pair`*2+1) transposed into a swizzled tile: tile row = column index, word `pair` of that row.
template <int G>
__device__ __forceinline__ void store_transposed_pair(uint32_t* tile, int col0, int pair, uint4 r0, uint4 r1) {
  const uint32_t a[4] = {r0.x, r0.y, r0.z, r0.w};
  const uint32_t b[4] = {r1.x, r1.y, r1.z, r1.w};
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const uint32_t lo = (a[q] & 0xffffu) | (b[q] << 16);
    const uint32_t hi = (a[q] >> 16) | (b[q] & 0xffff0000u);
    const int row_lo = col0 + 2 * q, row_hi = row_lo + 1;
    tile[row_lo * (4 * G) + swz<G>(row_lo, pair >> 2) * 4 + (pair & 3)] = lo;
    tile[row_hi * (4 * G) + swz<G>(row_hi, pair >> 2) * 4 + (pair & 3)] = hi;
  }
}
template <int G>
__device__ __forceinline__ uint4 load_swizzled_frag(const uint32_t* tile, int row, int group) {
  return *reinterpret_cast<const uint4*>(tile + row * (4 * G) + swz<G>(row, group) * 4);
}

}  // namespace
}  // namespace pd
