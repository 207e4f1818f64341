// Stand-alone momentum-SGD update into the version ring, for parameters whose gradient was
// materialised by another kernel:  m <- mu*m + g ;  w <- w_in - lr*m ;  ring <- bf16(w).
// Pure streaming work: per parameter it reads g, w, m (12 bytes) and writes w, m and the bf16 ring copy
// (10 bytes) in bf16 mode; in fp32 mode w_in is the ring slot of the latest version and w_out the next one.
#include "bf16_util.h"
#include "pd_kernels.h"

namespace pd {
namespace {


__global__ __launch_bounds__(256) void sgd_momentum_kernel(const float* __restrict__ g, const float* w_in,
                                                           float* w_out, float* __restrict__ mom,
                                                           bf16_t* __restrict__ ring, size_t n, float lr, float mu) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t n4 = n / 4;
  for (size_t i = tid; i < n4; i += stride) {
    const float4 gv = g ? reinterpret_cast<const float4*>(g)[i] : make_float4(0.f, 0.f, 0.f, 0.f);
    float4 m = reinterpret_cast<const float4*>(mom)[i];
    float4 w = reinterpret_cast<const float4*>(w_in)[i];
    m.x = mu * m.x + gv.x; m.y = mu * m.y + gv.y; m.z = mu * m.z + gv.z; m.w = mu * m.w + gv.w;
    w.x -= lr * m.x; w.y -= lr * m.y; w.z -= lr * m.z; w.w -= lr * m.w;
    reinterpret_cast<float4*>(mom)[i] = m;
    reinterpret_cast<float4*>(w_out)[i] = w;
    if (ring) {
      uint2 pk;
      pk.x = (uint32_t)f2bf(w.x) | ((uint32_t)f2bf(w.y) << 16);
      pk.y = (uint32_t)f2bf(w.z) | ((uint32_t)f2bf(w.w) << 16);
      reinterpret_cast<uint2*>(ring)[i] = pk;
    }
  }
  for (size_t i = n4 * 4 + tid; i < n; i += stride) {
    const float m = mu * mom[i] + (g ? g[i] : 0.f);
    const float w = w_in[i] - lr * m;
    mom[i] = m;
    w_out[i] = w;
    if (ring) ring[i] = f2bf(w);
  }
}

}  // namespace

hipError_t sgd_momentum_update(hipStream_t s, const float* g, const float* w_in, float* w_out, float* mom,
                               bf16_t* ring, size_t n, float lr, float mu, int grid_blocks) {
  if (n == 0) return hipSuccess;
  size_t blocks = (n / 4 + 255) / 256;
  const size_t cap = grid_blocks > 0 ? (size_t)grid_blocks : 8192;
  if (blocks > cap) blocks = cap;
  if (blocks < 1) blocks = 1;
  sgd_momentum_kernel<<<(unsigned)blocks, 256, 0, s>>>(g, w_in, w_out, mom, ring, n, lr, mu);
  return hipGetLastError();
}

}  // namespace pd
