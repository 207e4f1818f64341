// bfloat16 <-> float helpers shared by the device code (raw 16-bit storage, round to nearest even).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pd {

__device__ __forceinline__ uint16_t f2bf(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);  // keep NaN a NaN
  u += 0x7fffu + ((u >> 16) & 1u);                                             // nearest, ties to even
  return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf2f(uint16_t h) { return __uint_as_float(((uint32_t)h) << 16); }
__device__ __forceinline__ bool bf_positive(uint16_t h) { return (h & 0x8000u) == 0 && (h & 0x7fffu) != 0; }

}  // namespace pd
