// bf16 x bf16 -> fp32-accumulate GEMM kernels for gfx950 (CDNA4), built on the 32x32x16 bf16 MFMA.
//
// Three contractions of a Linear layer inside a pipeline stage:
//   forward   y  = act(x w^T + b)          reduction over in-features, both operands reduction-contiguous
//   dgrad     dx = (dz w) .* relu'         reduction over out-features, w is read "sideways"
//   wgrad+U   g  = dz^T x, then the momentum-SGD update of the fp32 master and the bf16 ring copy,
//             fused in one kernel so that the weight gradient never goes to HBM
//
// MFMA operand layout used throughout (wave = 64 lanes, lane l):
//   A fragment: row (l & 31) of a 32 x 16 block, reduction elements 8*(l >> 5) .. +7   (16 bytes)
//   B fragment: column (l & 31) of a 16 x 32 block, same reduction elements           (16 bytes)
//   D (16 floats): column (l & 31), rows 8*(r / 4) + 4*(l >> 5) + (r % 4) for r = 0..15
// A and B always take their 8 reduction elements from the same positions, so any fixed permutation
// of the reduction index inside an instruction cancels out.
#include "pd_kernels.h"

namespace pd {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ bf16x8 frag(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ __forceinline__ uint16_t f2bf(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);  // keep NaN a NaN
  u += 0x7fffu + ((u >> 16) & 1u);                                             // nearest, ties to even
  return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf2f(uint16_t h) { return __uint_as_float(((uint32_t)h) << 16); }
__device__ __forceinline__ bool bf_positive(uint16_t h) { return (h & 0x8000u) == 0 && (h & 0x7fffu) != 0; }

constexpr int kThreads = 256;
constexpr int BM = 64;    // rows of the output tile (minibatch direction)
constexpr int BN = 128;   // columns of the output tile
constexpr int BK = 64;    // reduction elements per LDS stage
constexpr int LDP = BK + 8;  // padded LDS row (bf16 elements) for reduction-contiguous tiles

__device__ __forceinline__ uint4 ldg16(const bf16_t* p) { return *reinterpret_cast<const uint4*>(p); }
__device__ __forceinline__ uint4 zero16() { return make_uint4(0u, 0u, 0u, 0u); }

// XOR swizzle of the 16-byte groups of a 128-byte LDS row holding 64 reduction elements of one output
// row/column.  Keeps both the transposing 4-byte writes and the 16-byte fragment reads spread over banks.
__device__ __forceinline__ int swz(int row, int group) { return group ^ (row & 7) ^ ((row >> 3) & 7); }

// Writes an 8-column x 2-row block (two 16-byte global chunks from consecutive reduction rows `pair`*2,
// `pair`*2+1) transposed into a swizzled tile: tile row = column index, word `pair` of that row.
__device__ __forceinline__ void store_transposed_pair(uint32_t* tile, int col0, int pair, uint4 r0, uint4 r1) {
  const uint32_t a[4] = {r0.x, r0.y, r0.z, r0.w};
  const uint32_t b[4] = {r1.x, r1.y, r1.z, r1.w};
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const uint32_t lo = (a[q] & 0xffffu) | (b[q] << 16);
    const uint32_t hi = (a[q] >> 16) | (b[q] & 0xffff0000u);
    const int row_lo = col0 + 2 * q, row_hi = row_lo + 1;
    tile[row_lo * 32 + swz(row_lo, pair >> 2) * 4 + (pair & 3)] = lo;
    tile[row_hi * 32 + swz(row_hi, pair >> 2) * 4 + (pair & 3)] = hi;
  }
}
__device__ __forceinline__ uint4 load_swizzled_frag(const uint32_t* tile, int row, int group) {
  return *reinterpret_cast<const uint4*>(tile + row * 32 + swz(row, group) * 4);
}

// ------------------------------------------------------------------------------------------------
// forward: partial or final y tile.  grid = (ceil(N/BN), ceil(M/BM), splits)
// ------------------------------------------------------------------------------------------------
template <bool DIRECT>
__global__ __launch_bounds__(kThreads) void gemm_nt_kernel(const bf16_t* __restrict__ X, const bf16_t* __restrict__ W,
                                                           const bf16_t* __restrict__ bias, bf16_t* __restrict__ Y,
                                                           float* __restrict__ Yf, float* __restrict__ ws, int M,
                                                           int N, int K, int relu, int splits) {
  __shared__ __attribute__((aligned(16))) bf16_t As[2][BM * LDP];
  __shared__ __attribute__((aligned(16))) bf16_t Bs[2][BN * LDP];
  const int t = threadIdx.x, l = t & 63, w = t >> 6;
  const int n0 = blockIdx.x * BN, m0 = blockIdx.y * BM, z = blockIdx.z;
  const int T = (K + BK - 1) / BK;
  const int kt0 = (int)((long long)z * T / splits), kt1 = (int)((long long)(z + 1) * T / splits);

  uint4 ra[2], rb[4];
  auto gload = [&](int kt) {
    const int k0 = kt * BK;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int c = t + kThreads * i, row = c >> 3, k = k0 + (c & 7) * 8, m = m0 + row;
      ra[i] = (m < M && k < K) ? ldg16(X + (size_t)m * K + k) : zero16();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int c = t + kThreads * i, row = c >> 3, k = k0 + (c & 7) * 8, n = n0 + row;
      rb[i] = (n < N && k < K) ? ldg16(W + (size_t)n * K + k) : zero16();
    }
  };
  auto sstore = [&](int buf) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int c = t + kThreads * i;
      *reinterpret_cast<uint4*>(&As[buf][(c >> 3) * LDP + (c & 7) * 8]) = ra[i];
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int c = t + kThreads * i;
      *reinterpret_cast<uint4*>(&Bs[buf][(c >> 3) * LDP + (c & 7) * 8]) = rb[i];
    }
  };

  f32x16 acc0 = {0}, acc1 = {0};
  if (kt0 < kt1) {
    gload(kt0);
    sstore(0);
    __syncthreads();
    for (int kt = kt0; kt < kt1; ++kt) {
      const int cur = (kt - kt0) & 1;
      if (kt + 1 < kt1) gload(kt + 1);
#pragma unroll
      for (int ks = 0; ks < BK / 16; ++ks) {
        const int kk = ks * 16 + (l >> 5) * 8;
        const uint4 b = *reinterpret_cast<const uint4*>(&Bs[cur][(32 * w + (l & 31)) * LDP + kk]);
        const uint4 a0 = *reinterpret_cast<const uint4*>(&As[cur][(l & 31) * LDP + kk]);
        const uint4 a1 = *reinterpret_cast<const uint4*>(&As[cur][(32 + (l & 31)) * LDP + kk]);
        acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(a0), frag(b), acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(a1), frag(b), acc1, 0, 0, 0);
      }
      if (kt + 1 < kt1) sstore(cur ^ 1);
      __syncthreads();
    }
  }

  const int n = n0 + 32 * w + (l & 31);
  if (n >= N) return;
  const float bv = (DIRECT && bias) ? bf2f(bias[n]) : 0.f;
#pragma unroll
  for (int blk = 0; blk < 2; ++blk) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int m = m0 + 32 * blk + 8 * (r >> 2) + 4 * (l >> 5) + (r & 3);
      if (m >= M) continue;
      const float v = blk ? acc1[r] : acc0[r];
      if (DIRECT) {
        float o = v + bv;
        if (relu) o = fmaxf(o, 0.f);
        if (Yf) Yf[(size_t)m * N + n] = o;
        else Y[(size_t)m * N + n] = f2bf(o);
      } else {
        ws[((size_t)z * M + m) * N + n] = v;
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// dgrad: dx tile = dz[M][N] * w[N][Kd], reduction over N.  grid = (ceil(Kd/BN), ceil(M/BM), splits)
// w rows are reduction rows here, so each 2x8 block of w is transposed on its way into LDS.
// ------------------------------------------------------------------------------------------------
template <bool DIRECT>
__global__ __launch_bounds__(kThreads) void gemm_nn_kernel(const bf16_t* __restrict__ dZ, const bf16_t* __restrict__ W,
                                                           const bf16_t* __restrict__ mask, bf16_t* __restrict__ dX,
                                                           float* __restrict__ ws, int M, int N, int Kd, int splits) {
  __shared__ __attribute__((aligned(16))) bf16_t As[2][BM * LDP];
  __shared__ __attribute__((aligned(16))) uint32_t Bt[2][BN * 32];
  const int t = threadIdx.x, l = t & 63, w = t >> 6;
  const int c0 = blockIdx.x * BN, m0 = blockIdx.y * BM, z = blockIdx.z;
  const int T = (N + BK - 1) / BK;
  const int rt0 = (int)((long long)z * T / splits), rt1 = (int)((long long)(z + 1) * T / splits);

  uint4 ra[2], rb0[2], rb1[2];
  auto gload = [&](int rt) {
    const int r0 = rt * BK;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int c = t + kThreads * i, row = c >> 3, n = r0 + (c & 7) * 8, m = m0 + row;
      ra[i] = (m < M && n < N) ? ldg16(dZ + (size_t)m * N + n) : zero16();
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int b = t + kThreads * i, kdc = b & 15, pair = b >> 4;
      const int n = r0 + 2 * pair, kd = c0 + 8 * kdc;
      rb0[i] = (n < N && kd < Kd) ? ldg16(W + (size_t)n * Kd + kd) : zero16();
      rb1[i] = (n + 1 < N && kd < Kd) ? ldg16(W + (size_t)(n + 1) * Kd + kd) : zero16();
    }
  };
  auto sstore = [&](int buf) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int c = t + kThreads * i;
      *reinterpret_cast<uint4*>(&As[buf][(c >> 3) * LDP + (c & 7) * 8]) = ra[i];
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int b = t + kThreads * i, kdc = b & 15, pair = b >> 4;
      store_transposed_pair(Bt[buf], 8 * kdc, pair, rb0[i], rb1[i]);
    }
  };

  f32x16 acc0 = {0}, acc1 = {0};
  if (rt0 < rt1) {
    gload(rt0);
    sstore(0);
    __syncthreads();
    for (int rt = rt0; rt < rt1; ++rt) {
      const int cur = (rt - rt0) & 1;
      if (rt + 1 < rt1) gload(rt + 1);
#pragma unroll
      for (int ks = 0; ks < BK / 16; ++ks) {
        const int kk = ks * 16 + (l >> 5) * 8;
        const uint4 b = load_swizzled_frag(Bt[cur], 32 * w + (l & 31), 2 * ks + (l >> 5));
        const uint4 a0 = *reinterpret_cast<const uint4*>(&As[cur][(l & 31) * LDP + kk]);
        const uint4 a1 = *reinterpret_cast<const uint4*>(&As[cur][(32 + (l & 31)) * LDP + kk]);
        acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(a0), frag(b), acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(a1), frag(b), acc1, 0, 0, 0);
      }
      if (rt + 1 < rt1) sstore(cur ^ 1);
      __syncthreads();
    }
  }

  const int kd = c0 + 32 * w + (l & 31);
  if (kd >= Kd) return;
#pragma unroll
  for (int blk = 0; blk < 2; ++blk) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int m = m0 + 32 * blk + 8 * (r >> 2) + 4 * (l >> 5) + (r & 3);
      if (m >= M) continue;
      const float v = blk ? acc1[r] : acc0[r];
      if (DIRECT) {
        uint16_t o = f2bf(v);
        if (mask && !bf_positive(mask[(size_t)m * Kd + kd])) o = 0;
        dX[(size_t)m * Kd + kd] = o;
      } else {
        ws[((size_t)z * M + m) * Kd + kd] = v;
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// split-K epilogue: sums the partial tiles in split order (deterministic), then bias/ReLU or ReLU-mask,
// rounds to bf16.  One thread per 4 consecutive columns.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void splitk_epilogue_kernel(const float* __restrict__ ws, int splits, int M, int N,
                                                              const bf16_t* __restrict__ bias,
                                                              const bf16_t* __restrict__ mask, int relu,
                                                              bf16_t* __restrict__ out, float* __restrict__ out_f) {
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t total4 = (size_t)M * N / 4;
  if (idx >= total4) return;
  const size_t e = idx * 4;
  const int n = (int)(e % N);
  float4 s = *reinterpret_cast<const float4*>(ws + e);
  for (int z = 1; z < splits; ++z) {
    const float4 p = *reinterpret_cast<const float4*>(ws + (size_t)z * M * N + e);
    s.x += p.x; s.y += p.y; s.z += p.z; s.w += p.w;
  }
  float v[4] = {s.x, s.y, s.z, s.w};
  uint16_t o[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    float x = v[j];
    if (bias) x += bf2f(bias[n + j]);
    if (relu) x = fmaxf(x, 0.f);
    v[j] = x;
    o[j] = f2bf(x);
    if (mask && !bf_positive(mask[e + j])) o[j] = 0;
  }
  if (out_f) {  // fp32 result (logits for the loss): no rounding, no mask
    *reinterpret_cast<float4*>(out_f + e) = make_float4(v[0], v[1], v[2], v[3]);
    return;
  }
  uint2 pk;
  pk.x = (uint32_t)o[0] | ((uint32_t)o[1] << 16);
  pk.y = (uint32_t)o[2] | ((uint32_t)o[3] << 16);
  *reinterpret_cast<uint2*>(out + e) = pk;
}

// ------------------------------------------------------------------------------------------------
// wgrad + momentum-SGD update.  One workgroup owns a TN x TK tile of w[N][K]:
//   phase 0  start the loads of the tile's fp32 master weights and momentum (they stay in registers
//            while the gradient tile is formed, which hides most of the HBM latency)
//   phase 1  g tile = dz[:, n-tile]^T x[:, k-tile], reducing over the minibatch rows in chunks of 64;
//            both operands are transposed into LDS on the way in
//   phase 2  g tile -> LDS (fp32), read back row-major so that every master / momentum / ring access
//            is a full-width contiguous row segment; m <- mu*m + g, w <- w - lr*m, ring <- bf16(w)
// grid.x = ceil(K/TK) * ceil(N/TN), k-tiles fastest.
// ------------------------------------------------------------------------------------------------
constexpr int TN = 64, TK = 128, MC = 64, GLD = TK + 4;
constexpr int kSlots = TN * TK / 4 / kThreads;  // float4 elements per thread in phase 2 (8)

__global__ __launch_bounds__(kThreads) void wgrad_update_kernel(
    const bf16_t* __restrict__ dZ, const bf16_t* __restrict__ X, float* __restrict__ master, float* __restrict__ mom,
    bf16_t* __restrict__ ring, float* __restrict__ master_b, float* __restrict__ mom_b, bf16_t* __restrict__ ring_b,
    int M, int N, int K, float lr, float mu) {
  __shared__ __attribute__((aligned(16))) uint32_t smem[TN * GLD];  // 33 KB; phase 1 uses the first 24 KB
  uint32_t* dZt = smem;             // [TN][32 words]  rows = n, 64 minibatch rows each
  uint32_t* Xt = smem + TN * 32;    // [TK][32 words]  rows = k
  float* G = reinterpret_cast<float*>(smem);

  const int t = threadIdx.x, l = t & 63, w = t >> 6;
  const int ktiles = (K + TK - 1) / TK;
  const int kt = blockIdx.x % ktiles, nt = blockIdx.x / ktiles;
  const int n0 = nt * TN, k0 = kt * TK;

  // phase 0: prefetch master and momentum of this thread's phase-2 elements
  float4 pw[kSlots], pm[kSlots];
#pragma unroll
  for (int q = 0; q < kSlots; ++q) {
    const int f = t + kThreads * q, row = f >> 5, k = k0 + (f & 31) * 4, n = n0 + row;
    if (n < N && k < K) {
      const size_t off = (size_t)n * K + k;
      pw[q] = *reinterpret_cast<const float4*>(master + off);
      pm[q] = *reinterpret_cast<const float4*>(mom + off);
    } else {
      pw[q] = make_float4(0.f, 0.f, 0.f, 0.f);
      pm[q] = pw[q];
    }
  }

  // phase 1
  f32x16 acc0 = {0}, acc1 = {0};
  for (int mc = 0; mc < M; mc += MC) {
    {
      const int nc = t & 7, pair = t >> 3;
      const int m = mc + 2 * pair, n = n0 + 8 * nc;
      const uint4 r0 = (m < M && n < N) ? ldg16(dZ + (size_t)m * N + n) : zero16();
      const uint4 r1 = (m + 1 < M && n < N) ? ldg16(dZ + (size_t)(m + 1) * N + n) : zero16();
      uint4 x0[2], x1[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int b = t + kThreads * i, kc = b & 15, p2 = b >> 4;
        const int mm = mc + 2 * p2, k = k0 + 8 * kc;
        x0[i] = (mm < M && k < K) ? ldg16(X + (size_t)mm * K + k) : zero16();
        x1[i] = (mm + 1 < M && k < K) ? ldg16(X + (size_t)(mm + 1) * K + k) : zero16();
      }
      if (mc) __syncthreads();  // previous chunk's fragments fully read
      store_transposed_pair(dZt, 8 * nc, pair, r0, r1);
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int b = t + kThreads * i, kc = b & 15, p2 = b >> 4;
        store_transposed_pair(Xt, 8 * kc, p2, x0[i], x1[i]);
      }
    }
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < MC / 16; ++ks) {
      const int g = 2 * ks + (l >> 5);
      const uint4 b = load_swizzled_frag(Xt, 32 * w + (l & 31), g);
      const uint4 a0 = load_swizzled_frag(dZt, (l & 31), g);
      const uint4 a1 = load_swizzled_frag(dZt, 32 + (l & 31), g);
      acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(a0), frag(b), acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(a1), frag(b), acc1, 0, 0, 0);
    }
  }
  __syncthreads();  // all fragment reads done before the tile memory is reused

  // phase 2a: accumulators -> LDS, G[n][k]
  {
    const int kcol = 32 * w + (l & 31);
#pragma unroll
    for (int blk = 0; blk < 2; ++blk) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int nrow = 32 * blk + 8 * (r >> 2) + 4 * (l >> 5) + (r & 3);
        G[nrow * GLD + kcol] = blk ? acc1[r] : acc0[r];
      }
    }
  }
  __syncthreads();

  // phase 2b: the update, row-major
#pragma unroll
  for (int q = 0; q < kSlots; ++q) {
    const int f = t + kThreads * q, row = f >> 5, c4 = (f & 31) * 4, k = k0 + c4, n = n0 + row;
    if (n < N && k < K) {
      const float4 g = *reinterpret_cast<const float4*>(&G[row * GLD + c4]);
      float4 m = pm[q], wv = pw[q];
      m.x = mu * m.x + g.x; m.y = mu * m.y + g.y; m.z = mu * m.z + g.z; m.w = mu * m.w + g.w;
      wv.x -= lr * m.x; wv.y -= lr * m.y; wv.z -= lr * m.z; wv.w -= lr * m.w;
      const size_t off = (size_t)n * K + k;
      *reinterpret_cast<float4*>(mom + off) = m;
      *reinterpret_cast<float4*>(master + off) = wv;
      uint2 pk;
      pk.x = (uint32_t)f2bf(wv.x) | ((uint32_t)f2bf(wv.y) << 16);
      pk.y = (uint32_t)f2bf(wv.z) | ((uint32_t)f2bf(wv.w) << 16);
      *reinterpret_cast<uint2*>(ring + off) = pk;
    }
  }

  // bias: column sums of dz in row order, by the workgroups of the first k-tile
  if (kt == 0 && master_b && t < TN) {
    const int n = n0 + t;
    if (n < N) {
      float g = 0.f;
      for (int m = 0; m < M; ++m) g += bf2f(dZ[(size_t)m * N + n]);
      const float mv = mu * mom_b[n] + g;
      const float bv = master_b[n] - lr * mv;
      mom_b[n] = mv;
      master_b[n] = bv;
      ring_b[n] = f2bf(bv);
    }
  }
}

int pick_splits(int tiles, int red_tiles) {
  int s = (512 + tiles - 1) / tiles;
  if (s > red_tiles / 2) s = red_tiles / 2;
  if (s > 32) s = 32;
  if (s < 1) s = 1;
  return s;
}

}  // namespace

size_t gemm_bf16_workspace_bytes(int M, int N, int K) {
  // fwd writes splits*M*N floats, dgrad splits*M*K floats; splits <= 32 and is 1 when there are >= 512 tiles.
  auto need = [](int rows, int cols, int red) {
    const int tiles = ((cols + BN - 1) / BN) * ((rows + BM - 1) / BM);
    const int s = pick_splits(tiles, (red + BK - 1) / BK);
    return s > 1 ? (size_t)s * rows * cols * sizeof(float) : (size_t)0;
  };
  const size_t a = need(M, N, K), b = need(M, K, N);
  return a > b ? a : b;
}

hipError_t linear_fwd_bf16(hipStream_t s, const bf16_t* x, const bf16_t* w, const bf16_t* b, bf16_t* y, float* y_f32,
                           int M, int N, int K, bool relu, float* ws, size_t ws_bytes) {
  const int tn = (N + BN - 1) / BN, tm = (M + BM - 1) / BM;
  int splits = pick_splits(tn * tm, (K + BK - 1) / BK);
  if (splits > 1 && (size_t)splits * M * N * sizeof(float) > ws_bytes) splits = 1;
  dim3 grid(tn, tm, splits);
  if (splits == 1) {
    gemm_nt_kernel<true><<<grid, kThreads, 0, s>>>(x, w, b, y, y_f32, nullptr, M, N, K, relu ? 1 : 0, 1);
  } else {
    gemm_nt_kernel<false><<<grid, kThreads, 0, s>>>(x, w, b, y, y_f32, ws, M, N, K, 0, splits);
    const size_t total4 = (size_t)M * N / 4;
    splitk_epilogue_kernel<<<(unsigned)((total4 + 255) / 256), 256, 0, s>>>(ws, splits, M, N, b, nullptr,
                                                                              relu ? 1 : 0, y, y_f32);
  }
  return hipGetLastError();
}

hipError_t linear_dgrad_bf16(hipStream_t s, const bf16_t* dz, const bf16_t* w, const bf16_t* mask, bf16_t* dx, int M,
                             int N, int K, float* ws, size_t ws_bytes) {
  const int tc = (K + BN - 1) / BN, tm = (M + BM - 1) / BM;
  int splits = pick_splits(tc * tm, (N + BK - 1) / BK);
  if (splits > 1 && (size_t)splits * M * K * sizeof(float) > ws_bytes) splits = 1;
  dim3 grid(tc, tm, splits);
  if (splits == 1) {
    gemm_nn_kernel<true><<<grid, kThreads, 0, s>>>(dz, w, mask, dx, nullptr, M, N, K, 1);
  } else {
    gemm_nn_kernel<false><<<grid, kThreads, 0, s>>>(dz, w, mask, dx, ws, M, N, K, splits);
    const size_t total4 = (size_t)M * K / 4;
    splitk_epilogue_kernel<<<(unsigned)((total4 + 255) / 256), 256, 0, s>>>(ws, splits, M, K, nullptr, mask, 0, dx,
                                                                              nullptr);
  }
  return hipGetLastError();
}

hipError_t linear_wgrad_update_bf16(hipStream_t s, const bf16_t* dz, const bf16_t* x, float* master_w, float* mom_w,
                                    bf16_t* ring_w, float* master_b, float* mom_b, bf16_t* ring_b, int M, int N, int K,
                                    float lr, float mu) {
  const unsigned tiles = (unsigned)(((K + TK - 1) / TK) * ((N + TN - 1) / TN));
  wgrad_update_kernel<<<tiles, kThreads, 0, s>>>(dz, x, master_w, mom_w, ring_w, master_b, mom_b, ring_b, M, N, K, lr,
                                                 mu);
  return hipGetLastError();
}

}  // namespace pd
