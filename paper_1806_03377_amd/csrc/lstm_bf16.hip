// Element-wise halves of an LSTM time step (the matrix halves are the GEMM kernels).  fp32 throughout;
// only the hidden state and the gate pre-activation gradients, which feed MFMA GEMMs, are rounded to bf16.
#include "bf16_util.h"
#include "mfma_util.h"
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


// ------------------------------------------------------------------------------------------------
// One recurrent step as ONE kernel: the skinny product with the recurrent weights and the cell update.  The
// product has few rows (the minibatch) and is read-once over a weight matrix that stays in L2, so what it costs is
// launches and latency, not flops: a workgroup owns a 16 x 16 tile of the output, its waves split the reduction
// range, every lane fetches its MFMA fragments (16 bytes, reduction-contiguous in both
// operands) straight from global memory, the waves' partial tiles are added in wave order through LDS, and the
// same threads then apply the gate non-linearities.
// ------------------------------------------------------------------------------------------------
// Uses the 16 x 16 x 32 MFMA (A fragment: row l & 15, reduction elements 8 (l >> 4) .. +7 of a 32-wide step; B
// fragment: column l & 15, same elements; D: column l & 15, rows 4 (l >> 4) + r for r = 0..3) so that a
// workgroup's tile is small and the launch has several workgroups per compute unit: these products are bound by
// memory latency, not by bandwidth or flops.
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Workgroups are dealt round-robin to the 8 XCDs, each with its own L2.  The recurrent weights are re-read at every
// time step, so the tiles are renumbered such that an XCD always works on the same contiguous range of hidden
// units (all row groups of a unit group together): its share of the weights (1/8) then stays in its L2 from
// step to step instead of every XCD streaming half of the matrix through a cache it does not fit in.
__device__ __forceinline__ void xcd_tile(int n_row_groups, int& unit_group, int& row_group) {
  const int total = gridDim.x, per = total >> 3;
  int id = blockIdx.x;
  if (id < per * 8) id = (id & 7) * per + (id >> 3);
  unit_group = id / n_row_groups;
  row_group = id - unit_group * n_row_groups;
}

// acc += A[row0 + (l & 15)][k0..k1) * brow[k0..k1)^T for one wave; k0, k1 multiples of 8.
template <int STEPS>
__device__ __forceinline__ void wave_skinny_gemm16(const bf16_t* __restrict__ arow /* this lane's A row or null */,
                                                   const bf16_t* __restrict__ brow /* this lane's B row or null */,
                                                   int k0, int k1, int l, f32x4& acc) {
  // STEPS reduction steps at a time: all their fragment loads are issued before the first MFMA, so the wave pays
  // the memory latency once per batch instead of once per step
  for (int kb = k0; kb < k1; kb += 32 * STEPS) {
    uint4 a[STEPS], b[STEPS];
#pragma unroll
    for (int st = 0; st < STEPS; ++st) {
      const int k = kb + 32 * st + 8 * (l >> 4);
      const bool live = k < k1;
      a[st] = (live && arow) ? ldg16(arow + k) : zero16();
      b[st] = (live && brow) ? ldg16(brow + k) : zero16();
    }
#pragma unroll
    for (int st = 0; st < STEPS; ++st)
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(frag(a[st]), frag(b[st]), acc, 0, 0, 0);
  }
}

// Forward: a workgroup owns 4 hidden units (their 4 x 4 = 16 gate columns) for 16 minibatch rows; grid =
// ceil(H / 4) * ceil(B / 16) workgroups (see xcd_tile); 4 waves split the reduction over H.
__global__ __launch_bounds__(256) void lstm_step_fwd_kernel(float* __restrict__ gates, const bf16_t* __restrict__ h_prev,
                                                            const bf16_t* __restrict__ whh,
                                                            const float* __restrict__ c_prev, float* __restrict__ c,
                                                            bf16_t* __restrict__ h, int B, int H) {
  __shared__ float red[4][16][17];
  const int t = threadIdx.x, l = t & 63, w = t >> 6;
  int ug, rg;
  xcd_tile((B + 15) / 16, ug, rg);
  const int u0 = ug * 4, r0 = rg * 16;
  const int kq = ((H + 127) / 128) * 32;  // reduction elements per wave (multiple of 32)
  const int k0 = w * kq, k1 = (k0 + kq) < H ? (k0 + kq) : H;
  const int cl = l & 15, unit = u0 + (cl & 3);
  const bf16_t* brow = unit < H ? whh + ((size_t)(cl >> 2) * H + unit) * H : nullptr;
  const bf16_t* arow = r0 + cl < B ? h_prev + (size_t)(r0 + cl) * H : nullptr;
  // the element-wise operands of this thread's (row, unit) are requested before the product, not after it
  const int erow = t >> 2, euu = t & 3;
  const bool eok = t < 64 && r0 + erow < B && u0 + euu < H;
  float gin[4] = {0.f, 0.f, 0.f, 0.f}, cprev = 0.f;
  if (eok) {
#pragma unroll
    for (int q = 0; q < 4; ++q) gin[q] = gates[(size_t)(r0 + erow) * 4 * H + q * H + u0 + euu];
    if (c_prev) cprev = c_prev[(size_t)(r0 + erow) * H + u0 + euu];
  }
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  if (k0 < k1) wave_skinny_gemm16<8>(arow, brow, k0, k1, l, acc);
#pragma unroll
  for (int r = 0; r < 4; ++r) red[w][4 * (l >> 4) + r][cl] = acc[r];
  __syncthreads();
  if (t < 64) {
    const int row = erow, uu = euu;
    const int b = r0 + row, j = u0 + uu;
    if (eok) {
      float a[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int col = q * 4 + uu;
        a[q] = gin[q] + (((red[0][row][col] + red[1][row][col]) + red[2][row][col]) + red[3][row][col]);
      }
      const float ig = sigmoidf(a[0]), fg = sigmoidf(a[1]), gg = tanhf(a[2]), og = sigmoidf(a[3]);
      const size_t idx = (size_t)b * H + j;
      const float cv = fg * cprev + ig * gg;
      const size_t e0 = (size_t)b * 4 * H + j;
      gates[e0] = ig; gates[e0 + H] = fg; gates[e0 + 2 * H] = gg; gates[e0 + 3 * H] = og;
      c[idx] = cv;
      h[idx] = f2bf(og * tanhf(cv));
    }
  }
}

// Backward: dh = dh_out + da_next * W_hh with W_hh^T stored [H][4H]; a workgroup owns 16 hidden units for 16
// minibatch rows; grid = ceil(H / 16) * ceil(B / 16) workgroups; 8 waves split the reduction over 4H.
__global__ __launch_bounds__(512) void lstm_step_bwd_kernel(const bf16_t* __restrict__ dh_out,
                                                            const bf16_t* __restrict__ da_next,
                                                            const bf16_t* __restrict__ whh_t, float* __restrict__ dc,
                                                            const float* __restrict__ gates, const float* __restrict__ c,
                                                            const float* __restrict__ c_prev, bf16_t* __restrict__ da,
                                                            int B, int H) {
  __shared__ float red[8][16][17];
  const int t = threadIdx.x, l = t & 63, w = t >> 6;
  int ug, rg;
  xcd_tile((B + 15) / 16, ug, rg);
  const int j0 = ug * 16, r0 = rg * 16;
  const int K = 4 * H;
  const int kq = ((K + 255) / 256) * 32;
  const int k0 = w * kq, k1 = (k0 + kq) < K ? (k0 + kq) : K;
  const int cl = l & 15;
  const bf16_t* brow = j0 + cl < H ? whh_t + (size_t)(j0 + cl) * K : nullptr;
  const bf16_t* arow = r0 + cl < B ? da_next + (size_t)(r0 + cl) * K : nullptr;
  // the element-wise operands of this thread's (row, unit) are requested before the product, not after it
  const int erow = (t >> 4) & 15, ecol = t & 15;
  const bool eok = t < 256 && r0 + erow < B && j0 + ecol < H;
  float ig = 0.f, fg = 0.f, gg = 0.f, og = 0.f, cc = 0.f, cp = 0.f, dcin = 0.f, dho = 0.f;
  if (eok) {
    const size_t idx = (size_t)(r0 + erow) * H + j0 + ecol, e0 = (size_t)(r0 + erow) * 4 * H + j0 + ecol;
    ig = gates[e0]; fg = gates[e0 + H]; gg = gates[e0 + 2 * H]; og = gates[e0 + 3 * H];
    cc = c[idx]; dcin = dc[idx];
    if (c_prev) cp = c_prev[idx];
    if (dh_out) dho = bf2f(dh_out[idx]);
  }
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  if (k0 < k1) wave_skinny_gemm16<16>(arow, brow, k0, k1, l, acc);  // 4H / 8 waves = 16 steps: one batch
#pragma unroll
  for (int r = 0; r < 4; ++r) red[w][4 * (l >> 4) + r][cl] = acc[r];
  __syncthreads();
  if (t < 256) {
    const int row = erow, col = ecol;
    const int b = r0 + row, j = j0 + col;
    if (eok) {
      float rec = 0.f;
#pragma unroll
      for (int q = 0; q < 8; ++q) rec += red[q][row][col];
      const size_t idx = (size_t)b * H + j;
      const float dh = dho + rec;
      const size_t e0 = (size_t)b * 4 * H + j;
      const float tc = tanhf(cc);
      const float dcv = dcin + dh * og * (1.f - tc * tc);
      da[e0] = f2bf(dcv * gg * ig * (1.f - ig));
      da[e0 + H] = f2bf(dcv * cp * fg * (1.f - fg));
      da[e0 + 2 * H] = f2bf(dcv * ig * (1.f - gg * gg));
      da[e0 + 3 * H] = f2bf(dh * tc * og * (1.f - og));
      dc[idx] = dcv * fg;
    }
  }
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

hipError_t lstm_step_forward(hipStream_t s, float* gates, const bf16_t* h_prev, const bf16_t* whh, const float* c_prev,
                             float* c, bf16_t* h, int B, int H) {
  if ((H % 8) || !h_prev) return hipErrorInvalidValue;
  lstm_step_fwd_kernel<<<((H + 3) / 4) * ((B + 15) / 16), 256, 0, s>>>(gates, h_prev, whh, c_prev, c, h, B, H);
  return hipGetLastError();
}

hipError_t lstm_step_backward(hipStream_t s, const bf16_t* dh_out, const bf16_t* da_next, const bf16_t* whh_t, float* dc,
                              const float* gates, const float* c, const float* c_prev, bf16_t* da, int B, int H) {
  if ((H % 8) || !da_next) return hipErrorInvalidValue;
  lstm_step_bwd_kernel<<<((H + 15) / 16) * ((B + 15) / 16), 512, 0, s>>>(dh_out, da_next, whh_t, dc, gates, c, c_prev,
                                                                       da, B, H);
  return hipGetLastError();
}

}  // namespace pd
