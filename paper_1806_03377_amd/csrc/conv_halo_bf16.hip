// 3x3, stride-1, pad-1 convolution (NHWC bf16, fp32 accumulate) that fetches its input ONCE per tile.
//
// The implicit-GEMM kernel (conv_dma_kernel) re-fetches a tile's input for each of the nine taps: 9 x 16 KB of
// activations per 256 pixels and 32 input channels through L2, the vector-memory path and LDS.  Here a workgroup owns
// an 8 x 32 patch of output pixels of one image; the 10 x 34 input pixels that patch needs (with its halo, zeros
// outside the image) are brought into LDS once per 64 input channels, 128 bytes per pixel, and every tap's MFMA operand
// is read from there at a shifted pixel index.  Only the weights are streamed per tap (BN filters x 64 channels =
// 8 or 16 KB, a ring of three or two such tiles).  Per MFMA that is a third (BN = 64) to less than half (BN = 128) of
// the bytes the implicit-GEMM kernel moves.
//
//   LDS     patch [352 pixel rows][128 bytes] (rows 340..351 never read) + weight ring [WR][BN rows][128 bytes];
//           a row's eight 16-byte slots are XOR-swizzled by ((row >> 1) & 7) (16 consecutive rows, which
//           one quarter of a 16-byte-per-lane read touches, then cover all 64 banks), applied on the global side of the direct
//           global -> LDS loads (lane L's chunk lands at M0 + 16 L: a wave-wide load fills 8 consecutive rows)
//   waves   four; BN = 64: wave w owns image rows 2w, 2w+1 of the patch (64 pixels) x 64 channels;
//           BN = 128: 2 x 2 waves of 4 image rows (128 pixels) x 64 channels
//   order   per 64-channel chunk: [barrier] patch -> LDS; per tap: wait for its weight tile, barrier (publishes it,
//           frees the slot of the tap before), request the tile WR-1 taps ahead, 4 reduction steps of MFMAs
//   two workgroups per compute unit (70 / 78 KB of LDS each), so that one computes while the other waits
//
// The same kernel serves the input gradient of such a layer (on dL/dy with flipped, transposed weights).
// Needs Ci % 64 == 0, 16-byte aligned tensors, sizes below 2^31 elements.
#include "bf16_util.h"
#include "mfma_util.h"
#include "pd_kernels.h"

namespace pd {
namespace {

__device__ __attribute__((aligned(16))) const uint32_t g_halo_zero[4] = {0u, 0u, 0u, 0u};
typedef __attribute__((address_space(3))) void halo_lds_void_t;

#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void halo_dma16(const bf16_t* lane_src, char* uniform_lds_dst) {
  const uint32_t lds_addr = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(halo_lds_void_t*)(uniform_lds_dst));
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(lane_src), "s"(lds_addr) : "memory", "m0");
}
#pragma clang diagnostic pop

constexpr int HT_H = 8, HT_W = 32, HP_W = HT_W + 2, HP_H = HT_H + 2, HP_PIX = HP_W * HP_H;  // 340 patch pixels
constexpr int HCC = 64, HROWB = HCC * 2;                  // input channels per chunk, bytes per LDS row
constexpr int HP_LOADS = 44, HP_ROWS = HP_LOADS * 8;      // wave-wide loads per patch (8 rows each), rows reserved
constexpr int HP_BYTES = HP_ROWS * HROWB;                 // 45056

__device__ __forceinline__ int halo_swz(int row) { return (row >> 1) & 7; }

template <int BN>
__global__ __launch_bounds__(256, 2) void conv3x3_halo_kernel(const bf16_t* __restrict__ X, const bf16_t* __restrict__ Wg,
                                                              ConvGeom g, ConvEpilogue ep, int tiles_x, int tiles_y,
                                                              int tiles_c) {
  constexpr int NWV = 4, WR = BN == 64 ? 3 : 2, WTILE = BN * HROWB;
  constexpr int WNW = BN / 64, WMW = NWV / WNW;          // waves along channels / image rows
  constexpr int NI = HT_H / WMW, NJ = 2;                 // 32-pixel rows and 32-channel blocks per wave
  constexpr int PQ = HP_LOADS / NWV;                     // patch loads per wave (11)
  constexpr int WQ = (BN / 8) / NWV;                     // weight-tile loads per wave (2 or 4)
  constexpr int KS = HCC / 16, MF = NI * NJ;
  constexpr int OLD = BN + 8;
  constexpr int kSmem = HP_BYTES + WR * WTILE;
  static_assert(kSmem >= HT_H * HT_W * OLD * 2, "the output staging area must fit");
  __shared__ __attribute__((aligned(1024))) char smem[kSmem];
  char* const wring = smem + HP_BYTES;
  const int t = threadIdx.x, l = t & 63;
  const int w = __builtin_amdgcn_readfirstlane(t >> 6), wm = w / WNW, wn = w % WNW;

  // tile of this workgroup: channel tiles of one pixel tile are neighbours (they read the same input), and an XCD
  // works on a contiguous run of tiles
  int id = blockIdx.x;
  {
    const int per = gridDim.x >> 3;
    if (id < per * 8) id = (id & 7) * per + (id >> 3);
  }
  const int tc = id % tiles_c;
  int rest = id / tiles_c;
  const int tx = rest % tiles_x;
  rest /= tiles_x;
  const int ty = rest % tiles_y, n = rest / tiles_y;
  const int co0 = tc * BN, x0 = tx * HT_W, y0 = ty * HT_H;
  const bf16_t* const zero = reinterpret_cast<const bf16_t*>(g_halo_zero);
  const int K9 = 9 * g.Ci, chunks = g.Ci / HCC;

  // patch loads: load number q * 4 + w covers patch rows 8 (q * 4 + w) .. + 7; this lane's pixel and channel group
  int poff[PQ];  // element offset of the lane's chunk for channel chunk 0, or -1 (outside the image / the patch)
#pragma unroll
  for (int q = 0; q < PQ; ++q) {
    const int pix = (q * NWV + w) * 8 + (l >> 3);
    const int py = pix / HP_W, px = pix - py * HP_W;
    const int iy = y0 - 1 + py, ix = x0 - 1 + px;
    const bool ok = pix < HP_PIX && (unsigned)iy < (unsigned)g.H && (unsigned)ix < (unsigned)g.W;
    poff[q] = ok ? ((n * g.H + iy) * g.W + ix) * g.Ci + 8 * ((l & 7) ^ halo_swz(pix)) : -1;
  }
  int woff[WQ];  // element offset of the lane's chunk of filter row co for tap 0, channel chunk 0, or -1
#pragma unroll
  for (int q = 0; q < WQ; ++q) {
    const int row = (q * NWV + w) * 8 + (l >> 3), co = co0 + row;
    woff[q] = co < g.Co ? co * K9 + 8 * ((l & 7) ^ halo_swz(row)) : -1;
  }
  auto load_patch = [&](int c) {
#pragma unroll
    for (int q = 0; q < PQ; ++q)
      halo_dma16(poff[q] >= 0 ? X + (poff[q] + c * HCC) : zero, smem + (q * NWV + w) * 1024);
  };
  auto load_wtile = [&](int q, int tau) {  // q-th load of the weight tile of global tap number tau = chunk * 9 + tap
    const int c = tau / 9, tap = tau - 9 * c;
    const bool ok = woff[q] >= 0 && c < chunks;
    halo_dma16(ok ? Wg + (woff[q] + tap * g.Ci + c * HCC) : zero, wring + (tau % WR) * WTILE + (q * NWV + w) * 1024);
  };

  // fragments.  A: output row r of the patch, lane's pixel (l & 31): patch pixel (r + dy) * 34 + (l & 31) + dx.
  // B: filter row.  Slot of reduction step ks, half h: (2 ks + h) ^ ((row >> 1) & 7).
  int apix[NI], fb[NJ];
#pragma unroll
  for (int i = 0; i < NI; ++i) apix[i] = (NI * wm + i) * HP_W + (l & 31);
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int row = 64 * wn + 32 * j + (l & 31);
    fb[j] = row * HROWB + (((l >> 5) ^ halo_swz(row)) << 4);
  }
  auto ldf = [&](const char* base, int o, int ks) { return *reinterpret_cast<const uint4*>(base + (o ^ (ks << 5))); };

  f32x16 acc[NI][NJ];
#pragma unroll
  for (int i = 0; i < NI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j) acc[i][j] = f32x16{0};

  // prologue: patch of chunk 0, weight tiles 0 .. WR-2
  load_patch(0);
#pragma unroll
  for (int d = 0; d < WR - 1; ++d)
#pragma unroll
    for (int q = 0; q < WQ; ++q) load_wtile(q, d);

  const int n_tau = 9 * chunks;
  int tap = 0, chunk = 0;
  for (int tau = 0; tau < n_tau; ++tau) {
    if (tap == 0 && chunk > 0) {
      // every wave is done with the previous chunk's patch; bring in this chunk's
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
      load_patch(chunk);
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    } else {
      // this wave's loads of tap tau's weight tile (and, for tau = 0, of the patch) have landed; the tile one tap
      // further (three-tile ring) may still be in flight
      asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"((WR - 2) * WQ) : "memory");
    }
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    // the slot of tap tau - 1 is free now: request tap tau + WR - 1 (past the end: zeros, never read)
    const char* wt = wring + (tau % WR) * WTILE;
    const int dy = tap / 3, dx = tap - 3 * dy, shift = dy * HP_W + dx;
    int fa[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int pix = apix[i] + shift;
      fa[i] = pix * HROWB + (((l >> 5) ^ halo_swz(pix)) << 4);
    }
    uint4 a[2][NI], b[2][NJ];
#pragma unroll
    for (int i = 0; i < NI; ++i) a[0][i] = ldf(smem, fa[i], 0);
#pragma unroll
    for (int j = 0; j < NJ; ++j) b[0][j] = ldf(wt, fb[j], 0);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int c = ks & 1, nx = c ^ 1;
      if (ks + 1 < KS) {
#pragma unroll
        for (int i = 0; i < NI; ++i) a[nx][i] = ldf(smem, fa[i], ks + 1);
#pragma unroll
        for (int j = 0; j < NJ; ++j) b[nx][j] = ldf(wt, fb[j], ks + 1);
      }
#pragma unroll
      for (int m = 0; m < MF; ++m) {
        const int i = m / NJ, j = m % NJ;
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(a[c][i]), frag(b[c][j]), acc[i][j], 0, 0, 0);
        if (m == 1 && ks < WQ) {  // one load of the tile WR-1 taps ahead behind the second MFMA of each step
          __builtin_amdgcn_sched_barrier(0);
          load_wtile(ks, tau + WR - 1);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
    if (++tap == 9) {
      tap = 0;
      ++chunk;
    }
  }
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
  __syncthreads();

  // bias / ReLU / rounding in registers, then through LDS so that global traffic is 16 bytes per lane
  bf16_t* ot = reinterpret_cast<bf16_t*>(smem);  // [256 pixels: image row of the patch * 32 + x][OLD]
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int cl = 64 * wn + 32 * j + (l & 31), cch = co0 + cl;
    const float bv = (ep.bias && cch < g.Co) ? bf2f(ep.bias[cch]) : 0.f;
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float v = acc[i][j][r] + bv;
        if (ep.relu) v = fmaxf(v, 0.f);
        ot[((NI * wm + i) * HT_W + 8 * (r >> 2) + 4 * (l >> 5) + (r & 3)) * OLD + cl] = f2bf(v);
      }
  }
  __syncthreads();
  constexpr int CPR = BN / 8;
#pragma unroll
  for (int i = 0; i < HT_H * HT_W * CPR / 256; ++i) {
    const int cidx = t + 256 * i, row = cidx / CPR, cc = cidx % CPR;
    const int oy = y0 + row / HT_W, ox = x0 + row % HT_W, co = co0 + cc * 8;
    if (oy >= g.Ho || ox >= g.Wo || co >= g.Co) continue;
    uint4 v = *reinterpret_cast<const uint4*>(&ot[row * OLD + cc * 8]);
    const size_t off = ((size_t)(n * g.Ho + oy) * g.Wo + ox) * g.Co + co;
    if (ep.mask) {
      const uint4 mk = ldg16(ep.mask + off);
      const uint32_t mw[4] = {mk.x, mk.y, mk.z, mk.w};
      uint32_t vw[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if (!bf_positive((uint16_t)(mw[q] & 0xffffu))) vw[q] &= 0xffff0000u;
        if (!bf_positive((uint16_t)(mw[q] >> 16))) vw[q] &= 0x0000ffffu;
      }
      v = make_uint4(vw[0], vw[1], vw[2], vw[3]);
    }
    *reinterpret_cast<uint4*>(ep.out + off) = v;
  }
}

bool g_conv_halo = true;

}  // namespace

int set_conv_halo(int on) {
  const int old = g_conv_halo ? 1 : 0;
  if (on == 0 || on == 1) g_conv_halo = on != 0;
  return old;
}

// Whether the halo kernel takes this convolution (3 x 3, stride 1, pad 1, plain input, 64-channel chunks).
bool conv3x3_halo_applies(const ConvGeom& g, const bf16_t* x, const bf16_t* w) {
  return g_conv_halo && g.kh == 3 && g.kw == 3 && g.stride == 1 && g.ph == 1 && g.pw == 1 && g.up <= 1 &&
         (g.Ci % HCC) == 0 && (g.Co % 8) == 0 && g.Ho == g.H && g.Wo == g.W &&
         ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(w)) & 15) == 0 &&
         (long long)g.N * g.H * g.W * g.Ci < (1ll << 31) && (long long)g.N * g.Ho * g.Wo * g.Co < (1ll << 31) &&
         (long long)g.Co * 9 * g.Ci < (1ll << 31);
}

hipError_t conv3x3_halo_bf16(hipStream_t s, const bf16_t* x, const bf16_t* w, const ConvGeom& g, const ConvEpilogue& ep) {
  const int tiles_x = (g.Wo + HT_W - 1) / HT_W, tiles_y = (g.Ho + HT_H - 1) / HT_H;
  if (g.Co <= 64) {
    conv3x3_halo_kernel<64><<<(unsigned)(g.N * tiles_y * tiles_x), 256, 0, s>>>(x, w, g, ep, tiles_x, tiles_y, 1);
  } else {
    const int tiles_c = (g.Co + 127) / 128;
    conv3x3_halo_kernel<128><<<(unsigned)(g.N * tiles_y * tiles_x * tiles_c), 256, 0, s>>>(x, w, g, ep, tiles_x, tiles_y,
                                                                                           tiles_c);
  }
  return hipGetLastError();
}

}  // namespace pd
