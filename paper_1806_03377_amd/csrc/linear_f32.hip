// fp32 Linear kernels (forward, dgrad, wgrad fused with the momentum-SGD update) for the all-fp32
// precision mode.  One generic 32x32-tile kernel with strided operands covers the three contractions;
// sums run over the reduction index in ascending order with fp32 FMAs, so results are deterministic.
// These shapes (a few hundred per side) are launch-latency bound; the kernel is kept simple.
#include "pd_kernels.h"

namespace pd {
namespace {

constexpr int T32 = 32;
enum { EPI_FWD = 0, EPI_DGRAD = 1, EPI_UPDATE = 2 };

struct EpiArgs {
  const float* bias;   // FWD: bias[j]
  int relu;            // FWD
  const float* mask;   // DGRAD: mask[i][j] > 0 keeps the value
  float* out;          // FWD / DGRAD output [I][J]
  const float* w_in;   // UPDATE
  float* w_out;
  float* mom;
  const float* b_in;
  float* b_out;
  float* mom_b;
  const float* dz;     // UPDATE: dz[M][N] for the bias column sums
  int M;
  UpdateRule rule;
};

// C[i][j] = sum_r A(i,r) B(r,j) with A(i,r) = a[i*a_is + r*a_rs], B(r,j) = b[r*b_rs + j*b_js]
// A workgroup owns a 32 x 32 tile of C and walks the reduction 128 elements at a time.  With a few workgroups on the
// whole chip the kernel's time is a sum of memory latencies, so every load of a step is issued unconditionally from
// a clamped address (out-of-range elements are replaced by zero afterwards, in registers), all thirty-two of a thread
// together, and the loads of step s+1 are in flight while step s is multiplied.
constexpr int TR = 128, NQ = T32 * TR / 256;  // reduction elements per step; elements per thread, operand and step
template <int EPI>
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ a, long a_is, long a_rs,
                                                       const float* __restrict__ b, long b_rs, long b_js, int I,
                                                       int J, int R, EpiArgs e) {
  __shared__ float As[T32][TR + 1];
  __shared__ float Bs[TR][T32 + 1];
  const int t = threadIdx.x, tx = t & 31, ty = t >> 5;
  const int i0 = blockIdx.y * T32, j0 = blockIdx.x * T32;
  // a thread's NQ elements of each operand tile; the fast thread index runs along whichever index is contiguous
  // in memory.  A tile: [32 i][TR r]; B tile: [TR r][32 j]
  const bool a_rc = a_rs == 1, b_jc = b_js == 1;
  const int a_i = a_rc ? (t / TR) : (t & 31), a_r = a_rc ? (t % TR) : (t >> 5);  // + (256 / TR) q (i) or + 8 q (r)
  const int b_r = b_jc ? (t >> 5) : (t % TR), b_j = b_jc ? (t & 31) : (t / TR);  // + 8 q (r) or + (256 / TR) q (j)
  const int a_di = a_rc ? 256 / TR : 0, a_dr = a_rc ? 0 : 8, b_dr = b_jc ? 8 : 0, b_dj = b_jc ? 0 : 256 / TR;
  float ra[NQ], rb[NQ];
  auto fetch = [&](int r0) {
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
      int i = i0 + a_i + a_di * q, r = r0 + a_r + a_dr * q;
      i = i < I ? i : I - 1;
      r = r < R ? r : R - 1;
      ra[q] = a[i * a_is + r * a_rs];
      int rr = r0 + b_r + b_dr * q, j = j0 + b_j + b_dj * q;
      rr = rr < R ? rr : R - 1;
      j = j < J ? j : J - 1;
      rb[q] = b[rr * b_rs + j * b_js];
    }
  };
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  fetch(0);
  for (int r0 = 0; r0 < R; r0 += TR) {
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
      const int ii = a_i + a_di * q, ar = a_r + a_dr * q, br = b_r + b_dr * q, jj = b_j + b_dj * q;
      As[ii][ar] = (i0 + ii < I && r0 + ar < R) ? ra[q] : 0.f;
      Bs[br][jj] = (r0 + br < R && j0 + jj < J) ? rb[q] : 0.f;
    }
    __syncthreads();
    if (r0 + TR < R) fetch(r0 + TR);  // (uniform; the values are first used after the next step's barrier)
    const int rn = R - r0 < TR ? R - r0 : TR;  // (zeros beyond the reduction's end are not multiplied)
#pragma unroll 8
    for (int r = 0; r < rn; ++r) {
      const float bv = Bs[r][tx];
#pragma unroll
      for (int q = 0; q < 4; ++q) acc[q] = fmaf(As[ty + 8 * q][r], bv, acc[q]);
    }
    __syncthreads();
  }
  const int j = j0 + tx;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int i = i0 + ty + 8 * q;
    if (i >= I || j >= J) continue;
    const size_t off = (size_t)i * J + j;
    if (EPI == EPI_FWD) {
      float v = acc[q] + (e.bias ? e.bias[j] : 0.f);
      if (e.relu) v = fmaxf(v, 0.f);
      e.out[off] = v;
    } else if (EPI == EPI_DGRAD) {
      e.out[off] = (e.mask && !(e.mask[off] > 0.f)) ? 0.f : acc[q];
    } else {
      if (e.rule.kind == kRuleGradOnly) {  // replicated stage: the sum over replicas comes first
        e.w_out[off] = acc[q];
        continue;
      }
      float m = e.mom[off], wv = e.w_in[off];
      apply_update(e.rule, acc[q], m, wv);
      e.mom[off] = m;
      e.w_out[off] = wv;
    }
  }
  if (EPI == EPI_UPDATE && blockIdx.x == 0 && e.b_in && t < T32) {
    const int n = i0 + t;  // rows of w are output features
    if (n < I) {
      float g = 0.f;
      for (int m = 0; m < e.M; ++m) g += e.dz[(size_t)m * I + n];
      if (e.rule.kind == kRuleGradOnly) {
        e.b_out[n] = g;
        return;
      }
      float mv = e.mom_b[n], bv = e.b_in[n];
      apply_update(e.rule, g, mv, bv);
      e.mom_b[n] = mv;
      e.b_out[n] = bv;
    }
  }
}

}  // namespace

hipError_t linear_fwd_f32(hipStream_t s, const float* x, const float* w, const float* b, float* y, int M, int N, int K,
                          bool relu) {
  if (M <= 0 || N <= 0 || K <= 0) return hipErrorInvalidValue;  // (the kernel clamps its addresses to the last element)
  EpiArgs e = {};
  e.bias = b; e.relu = relu ? 1 : 0; e.out = y;
  dim3 grid((N + T32 - 1) / T32, (M + T32 - 1) / T32);
  // y[m][n] = sum_k x[m][k] w[n][k]
  gemm_f32_kernel<EPI_FWD><<<grid, 256, 0, s>>>(x, K, 1, w, 1, K, M, N, K, e);
  return hipGetLastError();
}

hipError_t linear_dgrad_f32(hipStream_t s, const float* dz, const float* w, const float* mask, float* dx, int M, int N,
                            int K) {
  if (M <= 0 || N <= 0 || K <= 0) return hipErrorInvalidValue;  // (the kernel clamps its addresses to the last element)
  EpiArgs e = {};
  e.mask = mask; e.out = dx;
  dim3 grid((K + T32 - 1) / T32, (M + T32 - 1) / T32);
  // dx[m][k] = sum_n dz[m][n] w[n][k]
  gemm_f32_kernel<EPI_DGRAD><<<grid, 256, 0, s>>>(dz, N, 1, w, K, 1, M, K, N, e);
  return hipGetLastError();
}

hipError_t linear_wgrad_update_f32(hipStream_t s, const float* dz, const float* x, const float* w_in, float* w_out,
                                   float* mom_w, const float* b_in, float* b_out, float* mom_b, int M, int N, int K,
                                   UpdateRule rule) {
  if (M <= 0 || N <= 0 || K <= 0) return hipErrorInvalidValue;  // (the kernel clamps its addresses to the last element)
  EpiArgs e = {};
  e.w_in = w_in; e.w_out = w_out; e.mom = mom_w; e.b_in = b_in; e.b_out = b_out; e.mom_b = mom_b;
  e.dz = dz; e.M = M; e.rule = rule;
  dim3 grid((K + T32 - 1) / T32, (N + T32 - 1) / T32);
  // g[n][k] = sum_m dz[m][n] x[m][k]
  gemm_f32_kernel<EPI_UPDATE><<<grid, 256, 0, s>>>(dz, 1, N, x, K, 1, N, K, M, e);
  return hipGetLastError();
}

}  // namespace pd
