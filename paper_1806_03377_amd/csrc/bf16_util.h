// bfloat16 <-> float helpers shared by the device code (raw 16-bit storage, round to nearest even).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pd {

// fp32 -> bf16, nearest, ties to even, a NaN stays a NaN (quiet bit set, upper payload kept): gfx950's conversion
// instruction (v_cvt_pk_bf16_f32).  Checked against the integer formulation -- u += 0x7fff + ((u >> 16) & 1), NaNs
// (u >> 16) | 0x40 -- on all 2^32 bit patterns on an MI355X: identical, denormals and NaNs included; seven vector
// instructions fewer per value, which is what an epilogue over a short reduction mostly consists of.
__device__ __forceinline__ uint16_t f2bf(float f) { return __builtin_bit_cast(uint16_t, static_cast<__bf16>(f)); }
// two values into one register: low half a, high half b (one instruction)
typedef float bf_f32x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf_bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t f2bf_pair(float a, float b) {
  const bf_f32x2_t v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf_bf16x2_t));
}
__device__ __forceinline__ float bf2f(uint16_t h) { return __uint_as_float(((uint32_t)h) << 16); }
__device__ __forceinline__ bool bf_positive(uint16_t h) { return (h & 0x8000u) == 0 && (h & 0x7fffu) != 0; }

// An fp32 master weight kept as its bf16 rounding (which a weight-version ring holds anyway) plus the low 16 bits of
// its fp32 pattern.  Rounding to nearest even is an integer add on the pattern, so upper half = bf16 - carry, and
// the carry is 1 exactly when the low half is >= 0x8000 -- except for a tie that rounds down (low half 0x8000,
// upper half even), which would read back as a carry.  That one case is stored with low half 0x7fff: the master
// loses one fp32 unit in the last place there (a 2^-17 fraction of random values), and split/merge are exact inverses
// on everything they store.  NaNs are not preserved.
__device__ __forceinline__ void master_split1(float w, uint16_t& ring, uint16_t& rem) {
  const uint32_t u = __float_as_uint(w);
  ring = f2bf(w);
  uint16_t lo = (uint16_t)(u & 0xffffu);
  if (lo == 0x8000u && ring == (uint16_t)(u >> 16)) lo = 0x7fffu;  // tie rounded down
  rem = lo;
}
__device__ __forceinline__ float master_merge1(uint16_t ring, uint16_t rem) {
  const uint32_t up = (uint32_t)(uint16_t)(ring - (rem >= 0x8000u ? 1u : 0u));
  return __uint_as_float((up << 16) | rem);
}

// eight bf16 values <-> one 16-byte register quad
__device__ __forceinline__ void unpack8(uint4 v, uint16_t* o) {
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    o[2 * q] = (uint16_t)(w[q] & 0xffffu);
    o[2 * q + 1] = (uint16_t)(w[q] >> 16);
  }
}
__device__ __forceinline__ uint4 pack8(const uint16_t* o) {
  return make_uint4(o[0] | ((uint32_t)o[1] << 16), o[2] | ((uint32_t)o[3] << 16), o[4] | ((uint32_t)o[5] << 16),
                    o[6] | ((uint32_t)o[7] << 16));
}

}  // namespace pd
