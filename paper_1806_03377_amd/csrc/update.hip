// The update of a replicated stage (Section 3.3 round-robin replicas; Section 4: new parameters are handed out once
// the gradients of all replicas have been aggregated): the replicas leave their fp32 gradients of one round in
// separate buffers, and this kernel adds them up in replica order, takes the optimiser step on the one shared
// parameter state and writes the next slot of the version ring.
// Pure streaming work: per parameter it reads `count` gradients, w and the state (4*count + 8 bytes) and writes w,
// the state and, in bf16 mode, the ring copy (8 + 2 bytes).  In fp32 mode w_in is the ring slot of the latest
// version and w_out the next one; in bf16 mode w_in = w_out = the fp32 master copy.
#include "bf16_util.h"
#include "pd_kernels.h"

namespace pd {
namespace {

__global__ __launch_bounds__(256) void replica_sum_update_kernel(ReplicaGrads grads, const float* w_in, float* w_out,
                                                                 float* __restrict__ state, bf16_t* __restrict__ ring,
                                                                 size_t n, UpdateRule rule) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t n4 = n / 4;
  for (size_t i = tid; i < n4; i += stride) {
    float4 g = reinterpret_cast<const float4*>(grads.g[0])[i];
    for (int q = 1; q < grads.count; ++q) {
      const float4 h = reinterpret_cast<const float4*>(grads.g[q])[i];
      g.x += h.x; g.y += h.y; g.z += h.z; g.w += h.w;
    }
    float4 m = reinterpret_cast<const float4*>(state)[i];
    float4 w = reinterpret_cast<const float4*>(w_in)[i];
    apply_update(rule, g.x, m.x, w.x); apply_update(rule, g.y, m.y, w.y);
    apply_update(rule, g.z, m.z, w.z); apply_update(rule, g.w, m.w, w.w);
    reinterpret_cast<float4*>(state)[i] = m;
    reinterpret_cast<float4*>(w_out)[i] = w;
    if (ring) {
      uint2 pk;
      pk.x = (uint32_t)f2bf(w.x) | ((uint32_t)f2bf(w.y) << 16);
      pk.y = (uint32_t)f2bf(w.z) | ((uint32_t)f2bf(w.w) << 16);
      reinterpret_cast<uint2*>(ring)[i] = pk;
    }
  }
  for (size_t i = n4 * 4 + tid; i < n; i += stride) {
    float g = grads.g[0][i];
    for (int q = 1; q < grads.count; ++q) g += grads.g[q][i];
    float m = state[i], w = w_in[i];
    apply_update(rule, g, m, w);
    state[i] = m;
    w_out[i] = w;
    if (ring) ring[i] = f2bf(w);
  }
}

}  // namespace

hipError_t replica_sum_update(hipStream_t s, const ReplicaGrads& grads, const float* w_in, float* w_out, float* state,
                              bf16_t* ring, size_t n, UpdateRule rule) {
  if (n == 0) return hipSuccess;
  if (grads.count < 1 || grads.count > kMaxReplicas || rule.kind == kRuleGradOnly) return hipErrorInvalidValue;
  size_t blocks = (n / 4 + 255) / 256;
  if (blocks > 8192) blocks = 8192;  // 32 workgroups per compute unit; the loop strides over the rest
  if (blocks < 1) blocks = 1;
  replica_sum_update_kernel<<<(unsigned)blocks, 256, 0, s>>>(grads, w_in, w_out, state, ring, n, rule);
  return hipGetLastError();
}

}  // namespace pd
