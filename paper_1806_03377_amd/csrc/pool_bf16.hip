// General pooling (max / average, any window, stride and padding) and the channel-concatenation helpers of
// branched blocks, over NHWC bf16 tensors.  All of it is HBM-bound streaming work: 8 channels (16 bytes) per
// thread, consecutive threads on consecutive channel groups of a pixel.
#include "bf16_util.h"
#include "pd_kernels.h"

namespace pd {
namespace {

__device__ __forceinline__ uint4 ld16(const bf16_t* p) { return *reinterpret_cast<const uint4*>(p); }

// One thread per (output pixel, 8 channels).  Max: the first maximum in row-major window order is kept (the
// comparison is strict), padding is skipped.  Average: fp32 sum in row-major order over the positions inside the
// image, divided by k*k (padding counts as zeros).
// route (max pooling, window <= 4, optional): 8 bytes per thread, one per channel: bits 0-3 = the window position
// a * k + b of the first maximum, bit 4 = that maximum is positive, bit 5 = it is not a NaN.  pool2d_bwd_route_kernel
// needs nothing else of x and y.
template <bool MAX>
__global__ __launch_bounds__(256) void pool2d_fwd_kernel(const bf16_t* __restrict__ x, bf16_t* __restrict__ y,
                                                         uint2* __restrict__ route, PoolGeom g) {
  const int C8 = g.C / 8;
  const size_t total = (size_t)g.N * g.Ho * g.Wo * C8;
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int c8 = (int)(idx % C8);
  size_t q = idx / C8;
  const int wo = (int)(q % g.Wo);
  q /= g.Wo;
  const int ho = (int)(q % g.Ho);
  const size_t n = q / g.Ho;
  float acc[8];
  uint16_t best[8];
  uint32_t pos[8];
  bool have = false;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    acc[j] = 0.f;
    best[j] = 0;
    pos[j] = 0;
  }
  for (int a = 0; a < g.k; ++a) {
    const int hi = ho * g.stride - g.pad + a;
    if (hi < 0 || hi >= g.H) continue;
    for (int b = 0; b < g.k; ++b) {
      const int wi = wo * g.stride - g.pad + b;
      if (wi < 0 || wi >= g.W) continue;
      uint16_t v[8];
      unpack8(ld16(x + ((n * g.H + hi) * g.W + wi) * g.C + 8 * c8), v);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float f = bf2f(v[j]);
        if (MAX) {
          if (!have || f > acc[j]) {
            acc[j] = f;
            best[j] = v[j];
            pos[j] = (uint32_t)(a * g.k + b);
          }
        } else {
          acc[j] += f;
        }
      }
      have = true;
    }
  }
  if (!MAX) {
    const float inv = 1.f / (float)(g.k * g.k);
#pragma unroll
    for (int j = 0; j < 8; ++j) best[j] = f2bf(acc[j] * inv);
  }
  *reinterpret_cast<uint4*>(y + ((n * g.Ho + ho) * g.Wo + wo) * g.C + 8 * c8) = pack8(best);
  if (MAX && route) {
    uint32_t r[2] = {0u, 0u};
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const uint32_t code = (pos[j] & 15u) | (have && bf_positive(best[j]) ? 16u : 0u) | (have && acc[j] == acc[j] ? 32u : 0u);
      r[j >> 2] |= code << (8 * (j & 3));
    }
    route[idx] = make_uint2(r[0], r[1]);
  }
}

// Max pooling backward from the routing bytes: one thread per (input pixel, 8 channels) visits, in row-major order,
// the windows that cover its pixel and adds dy where the window's recorded position is this pixel (and the maximum
// was not a NaN and, with relu_mask, positive: the value at the recorded position IS the maximum).  Same sums in the
// same order as the comparing kernel below, without reading x or y.
__global__ __launch_bounds__(256) void pool2d_bwd_route_kernel(const uint2* __restrict__ route,
                                                               const bf16_t* __restrict__ dy, bf16_t* __restrict__ dx,
                                                               PoolGeom g, int relu_mask) {
  const int C8 = g.C / 8;
  const size_t total = (size_t)g.N * g.H * g.W * C8;
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int c8 = (int)(idx % C8);
  size_t q = idx / C8;
  const int wi = (int)(q % g.W);
  q /= g.W;
  const int hi = (int)(q % g.H);
  const size_t n = q / g.H;
  float acc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) acc[j] = 0.f;
  const int ho_hi = (hi + g.pad) / g.stride, wo_hi = (wi + g.pad) / g.stride;
  int ho_lo = hi + g.pad - g.k + 1, wo_lo = wi + g.pad - g.k + 1;
  ho_lo = ho_lo <= 0 ? 0 : (ho_lo + g.stride - 1) / g.stride;
  wo_lo = wo_lo <= 0 ? 0 : (wo_lo + g.stride - 1) / g.stride;
  const uint32_t need = relu_mask ? 48u : 32u;
  for (int ho = ho_lo; ho <= ho_hi && ho < g.Ho; ++ho)
    for (int wo = wo_lo; wo <= wo_hi && wo < g.Wo; ++wo) {
      const size_t oidx = ((n * g.Ho + ho) * g.Wo + wo) * C8 + c8;
      uint16_t dv[8];
      unpack8(ld16(dy + oidx * 8), dv);
      const uint2 r = route[oidx];
      const uint32_t me = (uint32_t)((hi - (ho * g.stride - g.pad)) * g.k + (wi - (wo * g.stride - g.pad)));
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const uint32_t code = ((j < 4 ? r.x : r.y) >> (8 * (j & 3))) & 255u;
        if ((code & 15u) == me && (code & need) == need) acc[j] += bf2f(dv[j]);
      }
    }
  uint16_t o[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) o[j] = f2bf(acc[j]);
  *reinterpret_cast<uint4*>(dx + ((n * g.H + hi) * g.W + wi) * g.C + 8 * c8) = pack8(o);
}

// Gather form of the backward pass: one thread per (input pixel, 8 channels) visits, in row-major order, the
// output windows that cover its pixel.  Average: adds dy/(k*k).  Max: adds dy where this pixel is the first
// position of the window (row-major) whose value equals the stored maximum.
template <bool MAX>
__global__ __launch_bounds__(256) void pool2d_bwd_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ y,
                                                         const bf16_t* __restrict__ dy, bf16_t* __restrict__ dx,
                                                         PoolGeom g, int relu_mask) {
  const int C8 = g.C / 8;
  const size_t total = (size_t)g.N * g.H * g.W * C8;
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int c8 = (int)(idx % C8);
  size_t q = idx / C8;
  const int wi = (int)(q % g.W);
  q /= g.W;
  const int hi = (int)(q % g.H);
  const size_t n = q / g.H;
  const size_t xoff = ((n * g.H + hi) * g.W + wi) * g.C + 8 * c8;
  uint16_t xv[8];
  if (MAX || relu_mask) unpack8(ld16(x + xoff), xv);
  float acc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) acc[j] = 0.f;
  // windows (ho, wo) with ho*stride - pad <= hi <= ho*stride - pad + k - 1
  const int ho_hi = (hi + g.pad) / g.stride, wo_hi = (wi + g.pad) / g.stride;
  int ho_lo = hi + g.pad - g.k + 1, wo_lo = wi + g.pad - g.k + 1;
  ho_lo = ho_lo <= 0 ? 0 : (ho_lo + g.stride - 1) / g.stride;
  wo_lo = wo_lo <= 0 ? 0 : (wo_lo + g.stride - 1) / g.stride;
  const float inv = 1.f / (float)(g.k * g.k);
  for (int ho = ho_lo; ho <= ho_hi && ho < g.Ho; ++ho)
    for (int wo = wo_lo; wo <= wo_hi && wo < g.Wo; ++wo) {
      const size_t yoff = ((n * g.Ho + ho) * g.Wo + wo) * g.C + 8 * c8;
      uint16_t dv[8];
      unpack8(ld16(dy + yoff), dv);
      if (!MAX) {
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] += bf2f(dv[j]) * inv;
        continue;
      }
      uint16_t yv[8];
      unpack8(ld16(y + yoff), yv);
      // does an earlier position of this window (row-major) already hold the maximum?
      bool earlier[8] = {false, false, false, false, false, false, false, false};
      const int a_me = hi - (ho * g.stride - g.pad), b_me = wi - (wo * g.stride - g.pad);
      for (int a = 0; a <= a_me; ++a) {
        const int h2 = ho * g.stride - g.pad + a;
        if (h2 < 0 || h2 >= g.H) continue;
        const int b_end = a == a_me ? b_me : g.k;
        for (int b = 0; b < b_end; ++b) {
          const int w2 = wo * g.stride - g.pad + b;
          if (w2 < 0 || w2 >= g.W) continue;
          uint16_t ov[8];
          unpack8(ld16(x + ((n * g.H + h2) * g.W + w2) * g.C + 8 * c8), ov);
#pragma unroll
          for (int j = 0; j < 8; ++j) earlier[j] = earlier[j] || bf2f(ov[j]) == bf2f(yv[j]);
        }
      }
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (!earlier[j] && bf2f(xv[j]) == bf2f(yv[j])) acc[j] += bf2f(dv[j]);
    }
  uint16_t o[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) o[j] = (relu_mask && !bf_positive(xv[j])) ? (uint16_t)0 : f2bf(acc[j]);
  *reinterpret_cast<uint4*>(dx + xoff) = pack8(o);
}

__global__ __launch_bounds__(256) void copy_channels_kernel(const bf16_t* __restrict__ src, int ld_src, int src_off,
                                                            bf16_t* __restrict__ dst, int ld_dst, int dst_off,
                                                            const bf16_t* __restrict__ mask, size_t pixels, int c8n) {
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= pixels * c8n) return;
  const size_t p = idx / c8n;
  const int c = (int)(idx - p * c8n) * 8;
  uint4 v = ld16(src + p * ld_src + src_off + c);
  const size_t doff = p * ld_dst + dst_off + c;
  if (mask) {
    uint16_t a[8], m[8];
    unpack8(v, a);
    unpack8(ld16(mask + doff), m);
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (!bf_positive(m[j])) a[j] = 0;
    v = pack8(a);
  }
  *reinterpret_cast<uint4*>(dst + doff) = v;
}

struct SumArgs {
  const bf16_t* src[kMaxBranches];
  int count;
};
__global__ __launch_bounds__(256) void sum_tensors_kernel(SumArgs a, const bf16_t* __restrict__ mask,
                                                          bf16_t* __restrict__ dst, size_t n8) {
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n8) return;
  float acc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) acc[j] = 0.f;
  for (int i = 0; i < a.count; ++i) {
    uint16_t v[8];
    unpack8(ld16(a.src[i] + idx * 8), v);
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] += bf2f(v[j]);
  }
  uint16_t o[8], m[8];
  if (mask) unpack8(ld16(mask + idx * 8), m);
#pragma unroll
  for (int j = 0; j < 8; ++j) o[j] = (mask && !bf_positive(m[j])) ? (uint16_t)0 : f2bf(acc[j]);
  *reinterpret_cast<uint4*>(dst + idx * 8) = pack8(o);
}

bool pool_geom_ok(const PoolGeom& g) {
  return g.N >= 1 && g.H >= 1 && g.W >= 1 && g.C >= 8 && (g.C % 8) == 0 && g.k >= 1 && g.stride >= 1 && g.pad >= 0 &&
         g.pad < g.k && g.Ho == (g.H + 2 * g.pad - g.k) / g.stride + 1 && g.Wo == (g.W + 2 * g.pad - g.k) / g.stride + 1 &&
         g.Ho >= 1 && g.Wo >= 1;
}

}  // namespace

bool pool2d_routes(bool is_max, const PoolGeom& g) { return is_max && g.k <= 4; }

hipError_t pool2d_forward_bf16(hipStream_t s, bool is_max, const bf16_t* x, bf16_t* y, void* route, const PoolGeom& g) {
  if (!pool_geom_ok(g)) return hipErrorInvalidValue;
  if (route && (!pool2d_routes(is_max, g) || (reinterpret_cast<uintptr_t>(route) & 7))) return hipErrorInvalidValue;
  const size_t total = (size_t)g.N * g.Ho * g.Wo * (g.C / 8);
  const unsigned blocks = (unsigned)((total + 255) / 256);
  if (is_max) pool2d_fwd_kernel<true><<<blocks, 256, 0, s>>>(x, y, static_cast<uint2*>(route), g);
  else pool2d_fwd_kernel<false><<<blocks, 256, 0, s>>>(x, y, nullptr, g);
  return hipGetLastError();
}

hipError_t pool2d_backward_routed_bf16(hipStream_t s, const void* route, const bf16_t* dy, bf16_t* dx, const PoolGeom& g,
                                       bool relu_mask) {
  if (!pool_geom_ok(g) || !pool2d_routes(true, g) || !route || (reinterpret_cast<uintptr_t>(route) & 7))
    return hipErrorInvalidValue;
  const size_t total = (size_t)g.N * g.H * g.W * (g.C / 8);
  pool2d_bwd_route_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>(static_cast<const uint2*>(route), dy, dx, g,
                                                                          relu_mask ? 1 : 0);
  return hipGetLastError();
}

hipError_t pool2d_backward_bf16(hipStream_t s, bool is_max, const bf16_t* x, const bf16_t* y, const bf16_t* dy,
                                bf16_t* dx, const PoolGeom& g, bool relu_mask) {
  if (!pool_geom_ok(g)) return hipErrorInvalidValue;
  const size_t total = (size_t)g.N * g.H * g.W * (g.C / 8);
  const unsigned blocks = (unsigned)((total + 255) / 256);
  if (is_max) pool2d_bwd_kernel<true><<<blocks, 256, 0, s>>>(x, y, dy, dx, g, relu_mask ? 1 : 0);
  else pool2d_bwd_kernel<false><<<blocks, 256, 0, s>>>(x, y, dy, dx, g, relu_mask ? 1 : 0);
  return hipGetLastError();
}

hipError_t copy_channels_bf16(hipStream_t s, const bf16_t* src, int ld_src, int src_off, bf16_t* dst, int ld_dst,
                              int dst_off, const bf16_t* mask, size_t pixels, int c) {
  if ((c % 8) || (ld_src % 8) || (ld_dst % 8) || (src_off % 8) || (dst_off % 8) || c < 8) return hipErrorInvalidValue;
  const size_t total = pixels * (c / 8);
  if (!total) return hipSuccess;
  copy_channels_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>(src, ld_src, src_off, dst, ld_dst, dst_off, mask,
                                                                       pixels, c / 8);
  return hipGetLastError();
}

hipError_t sum_tensors_bf16(hipStream_t s, const bf16_t* const* src, int count, const bf16_t* mask, bf16_t* dst,
                            size_t n) {
  if (count < 1 || count > kMaxBranches || (n % 8)) return hipErrorInvalidValue;
  SumArgs a;
  for (int i = 0; i < kMaxBranches; ++i) a.src[i] = i < count ? src[i] : nullptr;
  a.count = count;
  const size_t n8 = n / 8;
  if (!n8) return hipSuccess;
  sum_tensors_kernel<<<(unsigned)((n8 + 255) / 256), 256, 0, s>>>(a, mask, dst, n8);
  return hipGetLastError();
}

}  // namespace pd
