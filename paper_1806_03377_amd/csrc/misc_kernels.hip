// Element-wise helpers and the softmax cross-entropy loss of the output stage.
#include "bf16_util.h"
#include "pd_kernels.h"

namespace pd {
namespace {


__global__ __launch_bounds__(256) void copy_kernel(const uint8_t* __restrict__ src, uint8_t* __restrict__ dst,
                                                   size_t bytes, int vec_ok) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t done = 0;
  if (vec_ok) {
    const size_t n16 = bytes / 16;
    const uint4* s4 = reinterpret_cast<const uint4*>(src);
    uint4* d4 = reinterpret_cast<uint4*>(dst);
    for (size_t i = tid; i < n16; i += stride) d4[i] = s4[i];
    done = n16 * 16;
  }
  for (size_t i = done + tid; i < bytes; i += stride) dst[i] = src[i];
}

__global__ __launch_bounds__(256) void zero_kernel(uint32_t* __restrict__ dst, size_t words) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < words; i += stride) dst[i] = 0u;
}

// 16 bytes per lane; dst 16-byte aligned, `quads` pieces of four words
__global__ __launch_bounds__(256) void fill_pattern_kernel(uint4* __restrict__ dst, size_t quads, uint32_t value) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  const uint4 v = make_uint4(value, value, value, value);
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < quads; i += stride) dst[i] = v;
}

__global__ __launch_bounds__(256) void f32_to_bf16_kernel(const float* __restrict__ src, bf16_t* __restrict__ dst,
                                                          size_t n) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = f2bf(src[i]);
}
__global__ __launch_bounds__(256) void master_split_kernel(const float* __restrict__ master, bf16_t* __restrict__ ring,
                                                           uint16_t* __restrict__ rem, size_t n) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
    uint16_t r, lo;
    master_split1(master[i], r, lo);
    ring[i] = r;
    rem[i] = lo;
  }
}
__global__ __launch_bounds__(256) void master_merge_kernel(const bf16_t* __restrict__ ring,
                                                           const uint16_t* __restrict__ rem, float* __restrict__ master,
                                                           size_t n) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
    master[i] = master_merge1(ring[i], rem[i]);
}
__global__ __launch_bounds__(256) void bf16_to_f32_kernel(const bf16_t* __restrict__ src, float* __restrict__ dst,
                                                          size_t n) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = bf2f(src[i]);
}

__global__ __launch_bounds__(256) void transpose_kernel(const bf16_t* __restrict__ src, bf16_t* __restrict__ dst, int R,
                                                        int C) {
  __shared__ bf16_t tile[32][33];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  const int r0 = blockIdx.y * 32, c0 = blockIdx.x * 32;
  for (int i = ty; i < 32; i += 8)
    if (r0 + i < R && c0 + tx < C) tile[i][tx] = src[(size_t)(r0 + i) * C + c0 + tx];
  __syncthreads();
  for (int i = ty; i < 32; i += 8)
    if (c0 + i < C && r0 + tx < R) dst[(size_t)(c0 + i) * R + r0 + tx] = tile[tx][i];
}

template <bool BF>
__global__ __launch_bounds__(256) void relu_mask_kernel(const void* __restrict__ dy, const void* __restrict__ y,
                                                        void* __restrict__ dz, size_t n) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
    if (BF) {
      const uint16_t yv = static_cast<const uint16_t*>(y)[i];
      const bool pos = (yv & 0x8000u) == 0 && (yv & 0x7fffu) != 0;
      static_cast<uint16_t*>(dz)[i] = pos ? static_cast<const uint16_t*>(dy)[i] : (uint16_t)0;
    } else {
      static_cast<float*>(dz)[i] = static_cast<const float*>(y)[i] > 0.f ? static_cast<const float*>(dy)[i] : 0.f;
    }
  }
}

// Block-wide reductions in a fixed order (tree over 256 partials held in LDS).
__device__ __forceinline__ float block_reduce(float v, float* sh, bool is_max) {
  const int t = threadIdx.x;
  sh[t] = v;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if (t < s) sh[t] = is_max ? fmaxf(sh[t], sh[t + s]) : sh[t] + sh[t + s];
    __syncthreads();
  }
  const float r = sh[0];
  __syncthreads();
  return r;
}

// One workgroup per row: max, sum of exponentials, then dlogits = (p - onehot)/rows and the row's loss.
template <bool BF>
__global__ __launch_bounds__(256) void softmax_xent_kernel(const float* __restrict__ logits,
                                                           const int32_t* __restrict__ labels,
                                                           void* __restrict__ dlogits, float* __restrict__ row_loss,
                                                           int rows, int classes) {
  __shared__ float sh[256];
  const int r = blockIdx.x, t = threadIdx.x;
  const size_t base = (size_t)r * classes;
  auto ld = [&](int c) -> float { return logits[base + c]; };
  float mx = -INFINITY;
  for (int c = t; c < classes; c += 256) mx = fmaxf(mx, ld(c));
  mx = block_reduce(mx, sh, true);
  float sum = 0.f;
  for (int c = t; c < classes; c += 256) sum += expf(ld(c) - mx);
  sum = block_reduce(sum, sh, false);
  const float inv = 1.f / sum, invr = 1.f / (float)rows;
  int lab = labels[r];
  lab = lab < 0 ? 0 : (lab >= classes ? classes - 1 : lab);  // out-of-range labels are clamped, never dereferenced
  for (int c = t; c < classes; c += 256) {
    float d = expf(ld(c) - mx) * inv;
    if (c == lab) d -= 1.f;
    d *= invr;
    if (BF) static_cast<uint16_t*>(dlogits)[base + c] = f2bf(d);
    else static_cast<float*>(dlogits)[base + c] = d;
  }
  if (t == 0) row_loss[r] = logf(sum) + mx - ld(lab);
}

// The loss of a stage whose last Linear layer left split-K partial sums: logits = bias + sum over the partials (in
// split order), written out once (fp32) for the backward pass and for readers of the stage's output, and the
// softmax / cross-entropy of the row taken from registers in the same pass.  classes <= 256 * NV.
template <bool BF, int NV>
__global__ __launch_bounds__(256) void softmax_xent_partials_kernel(const float* __restrict__ part, int splits,
                                                                    const bf16_t* __restrict__ bias,
                                                                    float* __restrict__ logits,
                                                                    const int32_t* __restrict__ labels,
                                                                    void* __restrict__ dlogits, float* __restrict__ row_loss,
                                                                    int rows, int classes) {
  __shared__ float sh[256];
  const int r = blockIdx.x, t = threadIdx.x;
  const size_t base = (size_t)r * classes, stride = (size_t)rows * classes;
  int lab = labels[r];
  lab = lab < 0 ? 0 : (lab >= classes ? classes - 1 : lab);
  float v[NV];
  float mx = -INFINITY, zlab = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i) v[i] = 0.f;
  // Partial sums in split order.  A workgroup per row leaves few waves to hide the latency of dependent loads, so
  // the loads of eight splits are issued together and only then added; columns past the row read element 0 of the
  // row and are ignored later, splits past the last one re-read the last split and are multiplied by zero.
  for (int q0 = 0; q0 < splits; q0 += 8) {
    float p[8][NV];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int q = q0 + u < splits ? q0 + u : splits - 1;
      const float* src = part + (size_t)q * stride + base;
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const int c = t + 256 * i;
        p[u][i] = src[c < classes ? c : 0];
      }
    }
    __builtin_amdgcn_sched_barrier(0);  // all loads first: the scheduler otherwise pairs every load with its add
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const float keep = q0 + u < splits ? 1.f : 0.f;
#pragma unroll
      for (int i = 0; i < NV; ++i) v[i] = fmaf(keep, p[u][i], v[i]);
    }
  }
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = t + 256 * i;
    if (c < classes) {
      const float z = v[i] + (bias ? bf2f(bias[c]) : 0.f);
      logits[base + c] = z;
      v[i] = z;
      mx = fmaxf(mx, z);
      if (c == lab) zlab = z;
    }
  }
  mx = block_reduce(mx, sh, true);
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i)
    if (t + 256 * i < classes) {
      v[i] = expf(v[i] - mx);
      sum += v[i];
    }
  sum = block_reduce(sum, sh, false);
  const float inv = 1.f / sum, invr = 1.f / (float)rows;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = t + 256 * i;
    if (c < classes) {
      float d = v[i] * inv;
      if (c == lab) d -= 1.f;
      d *= invr;
      if (BF) static_cast<uint16_t*>(dlogits)[base + c] = f2bf(d);
      else static_cast<float*>(dlogits)[base + c] = d;
    }
  }
  if (lab % 256 == t) row_loss[r] = logf(sum) + mx - zlab;  // the thread that holds the label's logit
}

// The same for wide rows (a vocabulary): the row is read ONCE, 16 bytes per lane, and stays in registers
// (NV float4 per thread, classes <= 1024 NV) for the maximum, the sum and the result; bf16 results leave as 8-byte
// stores.  Needs classes % 4 == 0 and 16-byte aligned rows.
// e^x for x <= 0 (a logit minus its row maximum) as 2^(x log2 e) on the hardware exponential: two instructions
// where the library routine takes a dozen, which matters in a kernel that evaluates 30000 of them per row next to
// 0.9 GB of traffic.  Relative error below 1e-5 over the range that contributes to the sum (the product's rounding,
// |x| 2^-24, dominates); results under 2^-126 come out as zero.
__device__ __forceinline__ float exp_nonpos(float x) { return __builtin_amdgcn_exp2f(x * 1.44269504088896341f); }

template <bool BF, int NV>
__global__ __launch_bounds__(256) void softmax_xent_wide_kernel(const float* __restrict__ logits,
                                                                const int32_t* __restrict__ labels,
                                                                void* __restrict__ dlogits, float* __restrict__ row_loss,
                                                                int rows, int classes) {
  __shared__ float sh[256];
  const int r = blockIdx.x, t = threadIdx.x;
  const size_t base = (size_t)r * classes;
  const int nq = classes >> 2;  // float4 per row
  float4 v[NV];
  float mx = -INFINITY;
  // all of the row's loads first, unconditionally (a piece past the end re-reads the last one and is ignored):
  // a load under a condition, used right behind it, costs one memory latency per piece
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int q = t + 256 * i;
    v[i] = *reinterpret_cast<const float4*>(logits + base + 4 * (q < nq ? q : nq - 1));
  }
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int q = t + 256 * i;
    const float m4 = fmaxf(fmaxf(v[i].x, v[i].y), fmaxf(v[i].z, v[i].w));
    mx = q < nq ? fmaxf(mx, m4) : mx;
  }
  mx = block_reduce(mx, sh, true);
  int lab = labels[r];
  lab = lab < 0 ? 0 : (lab >= classes ? classes - 1 : lab);
  float sum = 0.f, zlab = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int q = t + 256 * i;
    if (q < nq) {
      if ((lab >> 2) == q) zlab = (lab & 3) == 0 ? v[i].x : (lab & 3) == 1 ? v[i].y : (lab & 3) == 2 ? v[i].z : v[i].w;
      v[i].x = exp_nonpos(v[i].x - mx); v[i].y = exp_nonpos(v[i].y - mx); v[i].z = exp_nonpos(v[i].z - mx); v[i].w = exp_nonpos(v[i].w - mx);
      sum += (v[i].x + v[i].y) + (v[i].z + v[i].w);
    }
  }
  sum = block_reduce(sum, sh, false);
  const float inv = 1.f / sum, invr = 1.f / (float)rows;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int q = t + 256 * i;
    if (q < nq) {
      float d[4] = {v[i].x * inv, v[i].y * inv, v[i].z * inv, v[i].w * inv};
      if ((lab >> 2) == q) d[lab & 3] -= 1.f;
#pragma unroll
      for (int e = 0; e < 4; ++e) d[e] *= invr;
      if (BF) {
        uint2 o;
        o.x = f2bf(d[0]) | ((uint32_t)f2bf(d[1]) << 16);
        o.y = f2bf(d[2]) | ((uint32_t)f2bf(d[3]) << 16);
        *reinterpret_cast<uint2*>(static_cast<uint16_t*>(dlogits) + base + 4 * q) = o;
      } else {
        *reinterpret_cast<float4*>(static_cast<float*>(dlogits) + base + 4 * q) = make_float4(d[0], d[1], d[2], d[3]);
      }
    }
  }
  if ((lab >> 2) % 256 == t) row_loss[r] = logf(sum) + mx - zlab;  // the thread that holds the label's logit
}

__global__ __launch_bounds__(256) void mean_kernel(const float* __restrict__ v, int n, float* __restrict__ out) {
  __shared__ float sh[256];
  float s = 0.f;
  for (int i = threadIdx.x; i < n; i += 256) s += v[i];
  s = block_reduce(s, sh, false);
  if (threadIdx.x == 0) *out = s / (float)n;
}

unsigned grid_for(size_t n) {
  size_t g = (n + 255) / 256;
  if (g > 4096) g = 4096;
  if (g < 1) g = 1;
  return (unsigned)g;
}

}  // namespace

hipError_t copy_bytes(hipStream_t s, const void* src, void* dst, size_t bytes) {
  if (bytes == 0) return hipSuccess;
  const int vec_ok = ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15u) == 0;
  copy_kernel<<<grid_for(bytes / 16 + 1), 256, 0, s>>>(static_cast<const uint8_t*>(src), static_cast<uint8_t*>(dst),
                                                       bytes, vec_ok);
  return hipGetLastError();
}
hipError_t fill_zero(hipStream_t s, void* dst, size_t bytes) {
  if (bytes == 0) return hipSuccess;
  zero_kernel<<<grid_for(bytes / 4), 256, 0, s>>>(static_cast<uint32_t*>(dst), bytes / 4);
  return hipGetLastError();
}
hipError_t fill_pattern16(hipStream_t s, void* dst, size_t bytes, uint32_t value) {
  if (bytes == 0) return hipSuccess;
  if ((bytes % 16) != 0 || (reinterpret_cast<uintptr_t>(dst) & 15) != 0) return hipErrorInvalidValue;
  fill_pattern_kernel<<<grid_for(bytes / 16), 256, 0, s>>>(static_cast<uint4*>(dst), bytes / 16, value);
  return hipGetLastError();
}
hipError_t f32_to_bf16(hipStream_t s, const float* src, bf16_t* dst, size_t n) {
  if (n == 0) return hipSuccess;
  f32_to_bf16_kernel<<<grid_for(n), 256, 0, s>>>(src, dst, n);
  return hipGetLastError();
}
hipError_t master_split(hipStream_t s, const float* master, bf16_t* ring, uint16_t* rem, size_t n) {
  if (n == 0) return hipSuccess;
  master_split_kernel<<<grid_for(n), 256, 0, s>>>(master, ring, rem, n);
  return hipGetLastError();
}
hipError_t master_merge(hipStream_t s, const bf16_t* ring, const uint16_t* rem, float* master, size_t n) {
  if (n == 0) return hipSuccess;
  master_merge_kernel<<<grid_for(n), 256, 0, s>>>(ring, rem, master, n);
  return hipGetLastError();
}
hipError_t transpose_bf16(hipStream_t s, const bf16_t* src, bf16_t* dst, int R, int C) {
  dim3 grid((C + 31) / 32, (R + 31) / 32);
  transpose_kernel<<<grid, 256, 0, s>>>(src, dst, R, C);
  return hipGetLastError();
}
hipError_t bf16_to_f32(hipStream_t s, const bf16_t* src, float* dst, size_t n) {
  if (n == 0) return hipSuccess;
  bf16_to_f32_kernel<<<grid_for(n), 256, 0, s>>>(src, dst, n);
  return hipGetLastError();
}
hipError_t relu_mask(hipStream_t s, const void* dy, const void* y, void* dz, size_t n, bool is_bf16) {
  if (n == 0) return hipSuccess;
  if (is_bf16) relu_mask_kernel<true><<<grid_for(n), 256, 0, s>>>(dy, y, dz, n);
  else relu_mask_kernel<false><<<grid_for(n), 256, 0, s>>>(dy, y, dz, n);
  return hipGetLastError();
}
hipError_t softmax_xent(hipStream_t s, const float* logits, const int32_t* labels, void* dlogits, float* row_loss,
                        float* loss, int rows, int classes, bool dlogits_bf16) {
  const bool aligned = (classes % 4) == 0 && ((reinterpret_cast<uintptr_t>(logits) | reinterpret_cast<uintptr_t>(dlogits)) & 15) == 0;
  if (aligned && classes > 2048 && classes <= 1024 * 32) {  // wide rows: one pass over the logits, row kept in registers
    if (dlogits_bf16) softmax_xent_wide_kernel<true, 32><<<rows, 256, 0, s>>>(logits, labels, dlogits, row_loss, rows, classes);
    else softmax_xent_wide_kernel<false, 32><<<rows, 256, 0, s>>>(logits, labels, dlogits, row_loss, rows, classes);
  } else if (dlogits_bf16) softmax_xent_kernel<true><<<rows, 256, 0, s>>>(logits, labels, dlogits, row_loss, rows, classes);
  else softmax_xent_kernel<false><<<rows, 256, 0, s>>>(logits, labels, dlogits, row_loss, rows, classes);
  if (loss) mean_kernel<<<1, 256, 0, s>>>(row_loss, rows, loss);
  return hipGetLastError();
}

hipError_t softmax_xent_partials(hipStream_t s, const float* part, int splits, const bf16_t* bias, float* logits,
                                 const int32_t* labels, void* dlogits, float* row_loss, float* loss, int rows,
                                 int classes, bool dlogits_bf16) {
  if (classes > kFusedLossMaxClasses || splits < 1) return hipErrorInvalidValue;
  if (dlogits_bf16)
    softmax_xent_partials_kernel<true, kFusedLossMaxClasses / 256><<<rows, 256, 0, s>>>(part, splits, bias, logits, labels, dlogits, row_loss, rows, classes);
  else
    softmax_xent_partials_kernel<false, kFusedLossMaxClasses / 256><<<rows, 256, 0, s>>>(part, splits, bias, logits, labels, dlogits, row_loss, rows, classes);
  if (loss) mean_kernel<<<1, 256, 0, s>>>(row_loss, rows, loss);
  return hipGetLastError();
}

}  // namespace pd
