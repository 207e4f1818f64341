// bf16 convolutions with a tiny reduction (kh*kw*Ci <= 32, at most 64 output channels): the first layer of an
// image network, e.g. 3x3 over 3 channels.  The taps of one output pixel become ONE 32-wide reduction row, so the
// forward pass is a [pixels] x [32] x [Co] product and the weight gradient a [Co] x [pixels] x [32] product.
// Both are bound by the traffic of the wide tensor (y or dz), not by arithmetic:
//   * the few input rows that 256 consecutive output pixels touch are staged in LDS with 16-byte loads, and the
//     per-pixel gather (27 two-byte reads for 3x3x3) runs against LDS instead of global memory;
//   * forward: the finished tile goes through LDS so that the output is written in 16-byte pieces;
//   * weight gradient: dz stays [pixel][channel] in LDS and the MFMA operands are fetched with the transposing
//     LDS read (ds_read_b64_tr_b16), the bias gradient comes from one more MFMA against a block of ones.
#include "bf16_util.h"
#include "mfma_util.h"
#include "pd_kernels.h"

namespace pd {
namespace {

constexpr int SK = 32, SLD = SK + 8;   // reduction width; padded row of the gathered tile (80 bytes)
constexpr int kRegion = 16 * 1024;     // bytes of input staged per 256 output pixels
typedef short v4i16_t __attribute__((ext_vector_type(4)));
typedef short v8i16_t __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) v4i16_t lds_v4i16_t;

__device__ __forceinline__ bf16x8 tr_frag(const char* lo, const char* hi) {
  const v4i16_t a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16_t*)lo);
  const v4i16_t b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16_t*)hi);
  const v8i16_t v = __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, v);
}

// Gathers the reduction rows of output pixels p0 .. p0+255 (one per thread) into tile[256][SLD].
// The input rows those pixels touch form one contiguous range of the NHWC tensor; if it fits, it is copied to
// `region` first (16-byte loads, the range widened to 16-byte boundaries) and the gather reads LDS.
// Contains two barriers; every thread of the workgroup must call it.
__device__ __forceinline__ void gather_tile(const bf16_t* __restrict__ X, const ConvGeom& g, long long p0, long long P,
                                            bf16_t* region, bf16_t* tile) {
  const int t = threadIdx.x;
  const long long total = (long long)g.N * g.H * g.W * g.Ci;
  // first and last pixel of the tile (workgroup-uniform)
  const long long pl = p0 + 255 < P ? p0 + 255 : P - 1;
  const long long r0 = p0 / g.Wo, r1 = pl / g.Wo;  // output rows counted over all images
  long long R0 = (r0 / g.Ho) * g.H + (r0 % g.Ho) * g.stride - g.ph;
  long long R1 = (r1 / g.Ho) * g.H + (r1 % g.Ho) * g.stride - g.ph + g.kh - 1;
  if (R0 < 0) R0 = 0;
  if (R1 > (long long)g.N * g.H - 1) R1 = (long long)g.N * g.H - 1;
  const long long e_lo = (R0 * g.W * g.Ci) & ~7ll;  // element range [e_lo, e_hi)
  const long long e_hi = (R1 + 1) * g.W * g.Ci;
  const bool staged = (e_hi - e_lo + 8) * 2 <= kRegion && (reinterpret_cast<uintptr_t>(X) & 15) == 0;
  if (staged) {
    const int chunks = (int)((e_hi - e_lo + 7) / 8);
    for (int c = t; c < chunks; c += kThreads) {
      const long long e = e_lo + 8ll * c;
      if (e + 8 <= total) {
        *reinterpret_cast<uint4*>(region + 8 * c) = ldg16(X + e);
      } else {
        for (int i = 0; i < 8; ++i) region[8 * c + i] = e + i < total ? X[e + i] : (bf16_t)0;
      }
    }
  }
  __syncthreads();
  const long long p = p0 + t;
  const bool live = p < P;
  int ho = 0, wo = 0;
  long long nrow = 0;
  if (live) {
    wo = (int)(p % g.Wo);
    const long long q = p / g.Wo;
    ho = (int)(q % g.Ho);
    nrow = (q / g.Ho) * g.H;
  }
  bf16_t* row = tile + t * SLD;
  if (staged && g.kh == 3 && g.kw == 3 && g.Ci == 3) {
    // The usual first layer: the 27 values are fetched with every index known at compile time, packed in registers
    // and written as four 16-byte pieces (rows 80 bytes apart: 16 consecutive lanes cover all banks) instead of 32
    // two-byte stores that meet four to a bank.
    const int hi0 = ho * g.stride - g.ph, wi0 = wo * g.stride - g.pw;
    const long long e00 = ((nrow + hi0) * g.W + wi0) * 3 - e_lo;  // region index of tap (0, 0), channel 0
    uint32_t v[32];
#pragma unroll
    for (int a = 0; a < 3; ++a) {
      const bool oka = live && (unsigned)(hi0 + a) < (unsigned)g.H;
#pragma unroll
      for (int b = 0; b < 3; ++b) {
        const bool ok = oka && (unsigned)(wi0 + b) < (unsigned)g.W;
        const int idx = ok ? (int)(e00 + (a * g.W + b) * 3) : 0;  // (a pixel outside the image reads element 0 and drops it)
#pragma unroll
        for (int c = 0; c < 3; ++c) v[(a * 3 + b) * 3 + c] = ok ? (uint32_t)region[idx + c] : 0u;
      }
    }
#pragma unroll
    for (int k = 27; k < 32; ++k) v[k] = 0u;
#pragma unroll
    for (int q = 0; q < 4; ++q)
      *reinterpret_cast<uint4*>(row + 8 * q) =
          make_uint4(v[8 * q] | (v[8 * q + 1] << 16), v[8 * q + 2] | (v[8 * q + 3] << 16),
                     v[8 * q + 4] | (v[8 * q + 5] << 16), v[8 * q + 6] | (v[8 * q + 7] << 16));
    __syncthreads();
    return;
  }
  int k = 0;
  for (int a = 0; a < g.kh; ++a) {
    const int hi = ho * g.stride - g.ph + a;
    for (int b = 0; b < g.kw; ++b) {
      const int wi = wo * g.stride - g.pw + b;
      const bool ok = live && (unsigned)hi < (unsigned)g.H && (unsigned)wi < (unsigned)g.W;
      const long long e = ((nrow + hi) * g.W + wi) * g.Ci;
      if (staged) {
        const bf16_t* src = region + (e - e_lo);
        for (int c = 0; c < g.Ci; ++c, ++k) row[k] = ok ? src[c] : (bf16_t)0;
      } else {
        const bf16_t* src = X + e;
        for (int c = 0; c < g.Ci; ++c, ++k) row[k] = ok ? src[c] : (bf16_t)0;
      }
    }
  }
  for (; k < SK; ++k) row[k] = 0;
  __syncthreads();
}

// Forward: 256 pixels x all Co <= 64 channels per workgroup; wave w owns pixels 64w .. 64w+63.
__global__ __launch_bounds__(kThreads) void conv_smallk_fwd_kernel(const bf16_t* __restrict__ X,
                                                                   const bf16_t* __restrict__ Wg, ConvGeom g,
                                                                   ConvEpilogue ep) {
  constexpr int OLD = 64 + 8;  // staged output row (elements)
  constexpr int kBytes = kRegion + 256 * SLD * 2 > 256 * OLD * 2 ? kRegion + 256 * SLD * 2 : 256 * OLD * 2;
  __shared__ __attribute__((aligned(16))) char smem[kBytes];
  __shared__ __attribute__((aligned(16))) bf16_t Bs[64 * SLD];
  __shared__ __attribute__((aligned(16))) float sbias[64];
  bf16_t* region = reinterpret_cast<bf16_t*>(smem);
  bf16_t* As = reinterpret_cast<bf16_t*>(smem + kRegion);
  const int t = threadIdx.x, l = t & 63, w = t >> 6;
  if (t < 64) sbias[t] = (ep.bias && t < g.Co) ? bf2f(ep.bias[t]) : 0.f;  // (published by gather_tile's barriers)
  const long long P = (long long)g.N * g.Ho * g.Wo;
  const long long p0 = (long long)blockIdx.x * 256;
  const int K = g.kh * g.kw * g.Ci;
  for (int e = t; e < 64 * SK; e += kThreads) {
    const int co = e / SK, k = e % SK;
    Bs[co * SLD + k] = (co < g.Co && k < K) ? Wg[(size_t)co * K + k] : (bf16_t)0;
  }
  gather_tile(X, g, p0, P, region, As);
  f32x16 acc[2][2] = {{f32x16{0}, f32x16{0}}, {f32x16{0}, f32x16{0}}};
#pragma unroll
  for (int ks = 0; ks < SK / 16; ++ks) {
    const int kk = ks * 16 + (l >> 5) * 8;
    uint4 a[2], b[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) a[i] = *reinterpret_cast<const uint4*>(&As[(64 * w + 32 * i + (l & 31)) * SLD + kk]);
#pragma unroll
    for (int j = 0; j < 2; ++j) b[j] = *reinterpret_cast<const uint4*>(&Bs[(32 * j + (l & 31)) * SLD + kk]);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(b[j]), frag(a[i]), acc[i][j], 0, 0, 0);
  }
  // (the filters are the MFMA's rows: acc[i][j][r] = channel 32 j + 8 (r >> 2) + 4 (l >> 5) + (r & 3) of pixel
  // 64 w + 32 i + (l & 31), runs of four channels per lane)
  if (ep.mask || (reinterpret_cast<uintptr_t>(ep.out) & 15)) {  // element-wise path (not used by the stage runtime)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int c = 32 * j + 8 * (r >> 2) + 4 * (l >> 5) + (r & 3);
          const long long p = p0 + 64 * w + 32 * i + (l & 31);
          if (c >= g.Co || p >= P) continue;
          float v = acc[i][j][r] + sbias[c];
          if (ep.relu) v = fmaxf(v, 0.f);
          uint16_t o = f2bf(v);
          const size_t off = (size_t)p * g.Co + c;
          if (ep.mask && !bf_positive(ep.mask[off])) o = 0;
          ep.out[off] = o;
        }
    return;
  }
  // bias, ReLU and rounding in registers, then through LDS: the 256 x Co tile is one contiguous piece of y
  __syncthreads();  // every wave is done reading As
  bf16_t* ot = reinterpret_cast<bf16_t*>(smem);  // [256][OLD]
  const float relu_floor = ep.relu ? 0.f : -__builtin_inff();
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const int ch = 32 * j + 8 * q4 + 4 * (l >> 5);
      const float4 b4 = *reinterpret_cast<const float4*>(&sbias[ch]);
      const float bv[4] = {b4.x, b4.y, b4.z, b4.w};
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        float v[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) v[r] = fmaxf(acc[i][j][4 * q4 + r] + bv[r], relu_floor);
        uint2 pk;
        pk.x = f2bf_pair(v[0], v[1]);
        pk.y = f2bf_pair(v[2], v[3]);
        *reinterpret_cast<uint2*>(&ot[(64 * w + 32 * i + (l & 31)) * OLD + ch]) = pk;
      }
    }
  __syncthreads();
  const int cpr = g.Co / 8;  // 16-byte pieces per pixel (Co % 8 == 0)
  for (int c = t; c < 256 * cpr; c += kThreads) {
    const int row = c / cpr, cc = c - row * cpr;
    if (p0 + row < P)
      *reinterpret_cast<uint4*>(ep.out + (size_t)(p0 + row) * g.Co + 8 * cc) =
          *reinterpret_cast<const uint4*>(&ot[row * OLD + 8 * cc]);
  }
}

// Weight gradient.  grid.x = splits; each workgroup walks chunks of 256 pixels; wave w reduces pixels
// 64w .. 64w+63 of every chunk into dW[co][k] (two 32x32 accumulators) and the bias gradient (dz against ones);
// the four waves' sums are added in wave order.  part[split][e] with e = co*K + k (K = kh*kw*Ci) for the weights
// and n_w + co for the bias.
__global__ __launch_bounds__(kThreads) void conv_smallk_wgrad_kernel(const bf16_t* __restrict__ dZ,
                                                                     const bf16_t* __restrict__ X,
                                                                     float* __restrict__ part, ConvGeom g,
                                                                     int chunks_per_split) {
  constexpr int kZ = 256 * 128;  // dz tile: [256 pixels][64 channels], the two 64-byte halves of a row swizzled
  constexpr int kLoop = kRegion + 256 * SLD * 2 + kZ, kRed = 4 * 64 * 33 * 4 + 4 * 64 * 4;
  __shared__ __attribute__((aligned(16))) char smem[kLoop > kRed ? kLoop : kRed];
  bf16_t* region = reinterpret_cast<bf16_t*>(smem);
  bf16_t* As = reinterpret_cast<bf16_t*>(smem + kRegion);
  char* Zs = smem + kRegion + 256 * SLD * 2;
  const int t = threadIdx.x, l = t & 63, w = t >> 6;
  const long long P = (long long)g.N * g.Ho * g.Wo;
  const int K = g.kh * g.kw * g.Ci;
  const long long nchunks_total = (P + 255) / 256;
  const long long chunk0 = (long long)blockIdx.x * chunks_per_split;
  long long chunk1 = chunk0 + chunks_per_split;
  if (chunk1 > nchunks_total) chunk1 = nchunks_total;
  f32x16 acc[2] = {f32x16{0}, f32x16{0}}, accb[2] = {f32x16{0}, f32x16{0}};  // [co block][k], [co block][any]
  const bf16x8 ones = __builtin_bit_cast(bf16x8, make_uint4(0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u));
  // transposing reads: this lane supplies pixel 8*(l>>5) + ((l>>2)&3) (+4 for the high half) and four channels
  const int pixl = 64 * w + 8 * (l >> 5) + ((l >> 2) & 3);
  const int chb = (16 * ((l >> 4) & 1) + 4 * (l & 3)) * 2;
  // dz of a chunk: 8 pieces of 16 bytes per pixel and thread, requested one chunk ahead (they arrive while the MFMAs
  // of the chunk before run: the wide tensor's memory latency is the one that matters here)
  uint4 zreg[8];
  auto fetch_dz = [&](long long ch) {
    const long long p0 = ch * 256;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int c = t + kThreads * i, r = c >> 3, pc = c & 7;
      const long long p = p0 + r;
      zreg[i] = (ch < chunk1 && p < P && 8 * pc < g.Co) ? ldg16(dZ + (size_t)p * g.Co + 8 * pc) : zero16();
    }
  };
  fetch_dz(chunk0);
  for (long long ch = chunk0; ch < chunk1; ++ch) {
    const long long p0 = ch * 256;
    // piece c of pixel r sits in 64-byte half (c/4) ^ ((r>>1)&1)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int c = t + kThreads * i, r = c >> 3, pc = c & 7;
      *reinterpret_cast<uint4*>(Zs + r * 128 + 64 * ((pc >> 2) ^ ((r >> 1) & 1)) + 16 * (pc & 3)) = zreg[i];
    }
    gather_tile(X, g, p0, P, region, As);  // (its barriers also publish Zs)
    fetch_dz(ch + 1);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const int r = pixl + 16 * ks;  // ((r >> 1) & 1) does not depend on ks or on the +4 of the high half
      const char* xb = reinterpret_cast<const char*>(As) + r * (SLD * 2) + chb;
      const bf16x8 b = tr_frag(xb, xb + 4 * SLD * 2);
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const char* zb = Zs + r * 128 + 64 * (i ^ ((r >> 1) & 1)) + chb;
        const bf16x8 a = tr_frag(zb, zb + 4 * 128);
        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
        accb[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, ones, accb[i], 0, 0, 0);
      }
    }
    __syncthreads();  // before the next chunk overwrites the tiles
  }
  // cross-wave reduction in wave order
  float* red = reinterpret_cast<float*>(smem);           // [4][64 * 33]
  float* bred = red + 4 * 64 * 33;                       // [4][64]
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int co = 32 * i + 8 * (r >> 2) + 4 * (l >> 5) + (r & 3);
      red[w * 64 * 33 + co * 33 + (l & 31)] = acc[i][r];
      if ((l & 31) == 0) bred[w * 64 + co] = accb[i][r];
    }
  __syncthreads();
  const size_t n_w = (size_t)g.Co * K;
  float* out = part + (size_t)blockIdx.x * (n_w + g.Co);
  for (int e = t; e < 64 * 32; e += kThreads) {
    const int co = e >> 5, k = e & 31, o = co * 33 + k;
    if (co < g.Co && k < K)
      out[(size_t)co * K + k] = ((red[o] + red[64 * 33 + o]) + red[2 * 64 * 33 + o]) + red[3 * 64 * 33 + o];
  }
  if (t < 64 && t < g.Co) out[n_w + t] = ((bred[t] + bred[64 + t]) + bred[128 + t]) + bred[192 + t];
}

}  // namespace

bool conv_is_smallk(const ConvGeom& g) { return g.kh * g.kw * g.Ci <= SK && g.Co <= 64; }

hipError_t conv_smallk_forward_bf16(hipStream_t s, const bf16_t* x, const bf16_t* w, const ConvGeom& g,
                                    const ConvEpilogue& ep) {
  if (!conv_is_smallk(g) || (g.Co % 8)) return hipErrorInvalidValue;
  const long long P = (long long)g.N * g.Ho * g.Wo;
  conv_smallk_fwd_kernel<<<(unsigned)((P + 255) / 256), kThreads, 0, s>>>(x, w, g, ep);
  return hipGetLastError();
}

hipError_t conv_smallk_wgrad_partial_bf16(hipStream_t s, const bf16_t* dz, const bf16_t* x, float* part, int splits,
                                          const ConvGeom& g) {
  if (!conv_is_smallk(g) || (g.Co % 8) || splits < 1) return hipErrorInvalidValue;
  if (reinterpret_cast<uintptr_t>(dz) & 15) return hipErrorInvalidValue;
  const long long P = (long long)g.N * g.Ho * g.Wo;
  const long long chunks = (P + 255) / 256;
  conv_smallk_wgrad_kernel<<<splits, kThreads, 0, s>>>(dz, x, part, g, (int)((chunks + splits - 1) / splits));
  return hipGetLastError();
}

}  // namespace pd
