// Element-wise halves of an LSTM time step (the matrix halves are the GEMM kernels).  fp32 throughout;
// only the hidden state and the gate pre-activation gradients, which feed MFMA GEMMs, are rounded to bf16.
#include "bf16_util.h"
#include "pd_kernels.h"

namespace pd {
namespace {

__device__ __forceinline__ float sigmoidf(float a) { return 1.f / (1.f + expf(-a)); }

__global__ __launch_bounds__(256) void lstm_cell_fwd_kernel(float* __restrict__ gates, const float* __restrict__ rec,
                                                            int splits, const float* __restrict__ c_prev,
                                                            float* __restrict__ c, bf16_t* __restrict__ h, int B,
                                                            int H) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= B * H) return;
  const int b = idx / H, j = idx - b * H;
  float a[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const size_t e = (size_t)b * 4 * H + q * H + j;
    float v = gates[e];
    for (int s = 0; s < splits; ++s) v += rec[(size_t)s * B * 4 * H + e];
    a[q] = v;
  }
  const float ig = sigmoidf(a[0]), fg = sigmoidf(a[1]), gg = tanhf(a[2]), og = sigmoidf(a[3]);
  const float cv = fg * (c_prev ? c_prev[idx] : 0.f) + ig * gg;
  const size_t e0 = (size_t)b * 4 * H + j;
  gates[e0] = ig; gates[e0 + H] = fg; gates[e0 + 2 * H] = gg; gates[e0 + 3 * H] = og;
  c[idx] = cv;
  h[idx] = f2bf(og * tanhf(cv));
}

__global__ __launch_bounds__(256) void lstm_cell_bwd_kernel(const bf16_t* __restrict__ dh_out,
                                                            const float* __restrict__ rec, int splits,
                                                            float* __restrict__ dc, const float* __restrict__ gates,
                                                            const float* __restrict__ c, const float* __restrict__ c_prev,
                                                            bf16_t* __restrict__ da, int B, int H) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= B * H) return;
  const int b = idx / H, j = idx - b * H;
  float dh = dh_out ? bf2f(dh_out[idx]) : 0.f;
  for (int s = 0; s < splits; ++s) dh += rec[(size_t)s * B * H + idx];
  const size_t e0 = (size_t)b * 4 * H + j;
  const float ig = gates[e0], fg = gates[e0 + H], gg = gates[e0 + 2 * H], og = gates[e0 + 3 * H];
  const float tc = tanhf(c[idx]);
  const float dcv = dc[idx] + dh * og * (1.f - tc * tc);
  const float cp = c_prev ? c_prev[idx] : 0.f;
  da[e0] = f2bf(dcv * gg * ig * (1.f - ig));
  da[e0 + H] = f2bf(dcv * cp * fg * (1.f - fg));
  da[e0 + 2 * H] = f2bf(dcv * ig * (1.f - gg * gg));
  da[e0 + 3 * H] = f2bf(dh * tc * og * (1.f - og));
  dc[idx] = dcv * fg;
}

}  // namespace

hipError_t lstm_cell_forward(hipStream_t s, float* gates, const float* rec_part, int splits, const float* c_prev, float* c,
                             bf16_t* h, int B, int H) {
  lstm_cell_fwd_kernel<<<(B * H + 255) / 256, 256, 0, s>>>(gates, rec_part, rec_part ? splits : 0, c_prev, c, h, B, H);
  return hipGetLastError();
}

hipError_t lstm_cell_backward(hipStream_t s, const bf16_t* dh_out, const float* rec_part, int splits, float* dc,
                              const float* gates, const float* c, const float* c_prev, bf16_t* da, int B, int H) {
  lstm_cell_bwd_kernel<<<(B * H + 255) / 256, 256, 0, s>>>(dh_out, rec_part, rec_part ? splits : 0, dc, gates, c, c_prev,
                                                            da, B, H);
  return hipGetLastError();
}

}  // namespace pd
