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
__device__ __forceinline__ void halo_dma16_at(const bf16_t* lane_src, uint32_t uniform_lds_addr) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(lane_src), "s"(uniform_lds_addr) : "memory", "m0");
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
  __shared__ __attribute__((aligned(16))) float sbias[BN];
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
  // (read in the epilogue, many barriers from here; fetched now so that nobody waits for it there)
  if (t < BN) sbias[t] = (ep.bias && co0 + t < g.Co) ? bf2f(ep.bias[co0 + t]) : 0.f;

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
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(b[c][j]), frag(a[c][i]), acc[i][j], 0, 0, 0);
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

  // bias / ReLU / rounding in registers, then through LDS so that global traffic is 16 bytes per lane.  The filters
  // are the MFMA's rows, so a lane holds runs of four channels of one pixel: acc[i][j][r] = channel 64 wn + 32 j +
  // 8 (r >> 2) + 4 (l >> 5) + (r & 3) of pixel (l & 31) in patch row NI wm + i, and a run goes to LDS as 8 bytes.
  bf16_t* ot = reinterpret_cast<bf16_t*>(smem);  // [256 pixels: image row of the patch * 32 + x][OLD]
  const float relu_floor = ep.relu ? 0.f : -__builtin_inff();
#pragma unroll
  for (int j = 0; j < NJ; ++j)
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const int ch = 64 * wn + 32 * j + 8 * q4 + 4 * (l >> 5);
      const float4 b4 = *reinterpret_cast<const float4*>(&sbias[ch]);
      const float bv[4] = {b4.x, b4.y, b4.z, b4.w};
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        float v[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) v[r] = fmaxf(acc[i][j][4 * q4 + r] + bv[r], relu_floor);
        uint2 pk;
        pk.x = f2bf_pair(v[0], v[1]);
        pk.y = f2bf_pair(v[2], v[3]);
        *reinterpret_cast<uint2*>(&ot[((NI * wm + i) * HT_W + (l & 31)) * OLD + ch]) = pk;
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

// ---- 64 input channels, at most 64 filters: the weights stay in registers and the workgroups stay on the chip ----
// With 64 filters a wave of the kernel above reads four 1-KB fragments from LDS for every four MFMAs, and the LDS pipe
// (128 bytes per clock and compute unit) is then busy exactly as long as the matrix pipes would be: the 64 -> 64 layer
// at 224 x 224 kept them busy in 27 % of the cycles.  (Hiding the memory latency alone -- the same persistent loop with
// the weights in LDS -- changed nothing: 356 against 354 us.)  Here every lane keeps its B operands of all 36 reduction
// steps (9 taps x 64 channels, 72 fragments = 288 registers; one wave per SIMD has 512) for the whole launch, loaded
// once from global memory; only the pixel fragments are read from LDS, half the bytes per MFMA.  A workgroup walks
// over its share of the tiles with two patch buffers: the patch of the next tile is requested before the MFMAs of
// this one start, so no tile but the first waits for memory, and there is no barrier between taps.  One workgroup per
// compute unit, grid = the number of compute units; an XCD's workgroups share a contiguous run of tiles (neighbouring
// tiles share halo pixels in that XCD's L2).
//   per tile: [barrier: the buffer to be refilled is no longer read] request the next patch; 36 reduction steps of
//   MFMAs; wait for the own requests, [barrier: the next patch is complete, this one no longer read]; outputs -> LDS
//   (over this tile's patch), [barrier], coalesced stores
__global__ __launch_bounds__(256, 1) void conv3x3_halo_resident_kernel(const bf16_t* __restrict__ X,
                                                                       const bf16_t* __restrict__ Wg, ConvGeom g,
                                                                       ConvEpilogue ep, int tiles_x, int tiles_y) {
  constexpr int NWV = 4, BN = 64, NI = 2, NJ = 2, PQ = HP_LOADS / NWV, KS = HCC / 16;
  constexpr int OLD = BN + 8;
  static_assert(HP_BYTES >= HT_H * HT_W * OLD * 2, "the output staging area must fit");
  __shared__ __attribute__((aligned(1024))) char smem[2 * HP_BYTES];
  __shared__ __attribute__((aligned(16))) float sbias[BN];
  const int t = threadIdx.x, l = t & 63;
  const int w = __builtin_amdgcn_readfirstlane(t >> 6);
  const uint32_t lds_base = lds_address_of(smem);
  if (t < BN) sbias[t] = (ep.bias && t < g.Co) ? bf2f(ep.bias[t]) : 0.f;  // (published by the first tile's barrier)
  const bf16_t* const zero = reinterpret_cast<const bf16_t*>(g_halo_zero);
  const int K9 = 9 * HCC;

  // this workgroup's tiles: XCD x (workgroups x, x + 8, ...) owns tiles [lo, hi); its j-th workgroup takes lo + j,
  // lo + j + per_x, ...
  const int n_tiles = g.N * tiles_y * tiles_x;
  const int xcd = blockIdx.x & 7, per_x = gridDim.x >> 3;
  const int lo = (int)((long long)xcd * n_tiles / 8), hi = (int)((long long)(xcd + 1) * n_tiles / 8);
  int tile = lo + (int)(blockIdx.x >> 3);
  if (tile >= hi) return;

  // patch loads: load number q * 4 + w covers patch rows 8 (q * 4 + w) .. + 7.  Rows 340..351 are never read: their
  // lanes fetch the patch's last pixel again.
  int prel[PQ];  // element offset of this lane's chunk from the patch's pixel (0, 0)
#pragma unroll
  for (int q = 0; q < PQ; ++q) {
    const int pix0 = (q * NWV + w) * 8 + (l >> 3), pix = pix0 < HP_PIX ? pix0 : HP_PIX - 1;
    const int py = pix / HP_W, px = pix - py * HP_W;
    prel[q] = (py * g.W + px) * HCC + 8 * ((l & 7) ^ halo_swz(pix0));
  }
  // the q-th load of this wave for the patch of the tile at image n, pixel (y0, x0), into buffer buf.  base: element
  // offset of the patch's pixel (0, 0) = image pixel (y0 - 1, x0 - 1) (outside the image for border tiles, where it is
  // only used for pixels that lie inside); inside: the whole patch lies inside the image
  auto load_patch_one = [&](int q, int buf, long long base, int y0, int x0, bool inside) {
    const uint32_t dst = lds_base + (uint32_t)(buf * HP_BYTES + (q * NWV + w) * 1024);
    if (inside) {
      halo_dma16_at(X + (base + prel[q]), dst);
    } else {
      const int pix0 = (q * NWV + w) * 8 + (l >> 3), pix = pix0 < HP_PIX ? pix0 : HP_PIX - 1;
      const int py = pix / HP_W, iy = y0 - 1 + py, ix = x0 - 1 + (pix - py * HP_W);
      const bool ok = (unsigned)iy < (unsigned)g.H && (unsigned)ix < (unsigned)g.W;
      halo_dma16_at(ok ? X + (base + prel[q]) : zero, dst);
    }
  };
  auto tile_origin = [&](int tl, int& n, int& y0, int& x0) {
    const int tx = tl % tiles_x, r = tl / tiles_x, ty = r % tiles_y;
    n = r / tiles_y; y0 = ty * HT_H; x0 = tx * HT_W;
  };
  auto patch_base = [&](int n, int y0, int x0) { return (((long long)n * g.H + (y0 - 1)) * g.W + (x0 - 1)) * HCC; };
  auto patch_inside = [&](int y0, int x0) { return y0 >= 1 && x0 >= 1 && y0 + HT_H < g.H && x0 + HT_W < g.W; };
  // A operands of the MFMAs (the matrix rows = output channels): filter 32 j + (l & 31), reduction elements
  // 16 ks + 8 (l >> 5) .. + 7 of every tap (zeros past Co)
  uint4 bw[9][KS][NJ];
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int co = 32 * j + (l & 31);
    const bf16_t* wrow = Wg + (co * K9 + 8 * (l >> 5));
#pragma unroll
    for (int tap = 0; tap < 9; ++tap)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) bw[tap][ks][j] = co < g.Co ? ldg16(wrow + tap * HCC + 16 * ks) : zero16();
  }
  {
    int n, y0, x0;
    tile_origin(tile, n, y0, x0);
    const long long base = patch_base(n, y0, x0);
    const bool inside = patch_inside(y0, x0);
#pragma unroll
    for (int q = 0; q < PQ; ++q) load_patch_one(q, 0, base, y0, x0, inside);
  }

  // B operands (the matrix columns = pixels): output row r of the patch, lane's pixel (l & 31), tap (dy, dx): patch
  // pixel (r + dy) * 34 + (l & 31) + dx.  Slot of reduction step ks, half h: (2 ks + h) ^ ((pixel >> 1) & 7).
  int fa[9][NI];
#pragma unroll
  for (int tap = 0; tap < 9; ++tap)
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int pix = (NI * w + i + tap / 3) * HP_W + (l & 31) + tap % 3;
      fa[tap][i] = pix * HROWB + (((l >> 5) ^ halo_swz(pix)) << 4);
    }
  auto ldf = [&](const char* base, int o, int ks) { return *reinterpret_cast<const uint4*>(base + (o ^ (ks << 5))); };
  const float relu_floor = ep.relu ? 0.f : -__builtin_inff();

  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");  // the first patch; the bias values' LDS stores
  for (int it = 0;; ++it) {
    const int cur = it & 1;
    const int next_tile = tile + per_x;
    const bool has_next = next_tile < hi;
    char* const patch = smem + cur * HP_BYTES;
    // first tile: publishes the patch; later: every wave has left the previous tile's staging area, which is
    // the buffer the next patch goes to
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    // the next tile's patch is requested from inside the MFMA loop below, one load every third reduction step (the
    // address arithmetic and the issue then cost nothing: the wave is waiting for the matrix pipe there anyway)
    int nn, ny0, nx0;
    tile_origin(has_next ? next_tile : tile, nn, ny0, nx0);
    const long long nbase = patch_base(nn, ny0, nx0);
    const bool ninside = patch_inside(ny0, nx0);

    // acc[i][j][r]: channel 32 j + 8 (r >> 2) + 4 (l >> 5) + (r & 3) of pixel (l & 31) in patch row NI w + i
    f32x16 acc[NI][NJ];
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
      for (int j = 0; j < NJ; ++j) acc[i][j] = f32x16{0};
    uint4 a[3][NI];  // fragments of this step and the next two
#pragma unroll
    for (int i = 0; i < NI; ++i) a[0][i] = ldf(patch, fa[0][i], 0);
#pragma unroll
    for (int i = 0; i < NI; ++i) a[1][i] = ldf(patch, fa[0][i], 1);
#pragma unroll
    for (int s36 = 0; s36 < 9 * KS; ++s36) {
      // (the scheduler, short of registers, would otherwise move each read down to just before its first use)
      if (s36 + 2 < 9 * KS) {
#pragma unroll
        for (int i = 0; i < NI; ++i) a[(s36 + 2) % 3][i] = ldf(patch, fa[(s36 + 2) / KS][i], (s36 + 2) % KS);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int i = 0; i < NI; ++i)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(bw[s36 / KS][s36 % KS][j]), frag(a[s36 % 3][i]), acc[i][j], 0, 0, 0);
      if (s36 % 3 == 1 && s36 / 3 < PQ && has_next) load_patch_one(s36 / 3, cur ^ 1, nbase, ny0, nx0, ninside);
      __builtin_amdgcn_sched_barrier(0);
    }
    // this wave's requests for the next patch have landed and its reads of this one are done; after the barrier that
    // holds for every wave
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");

    // bias / ReLU / rounding in registers (a lane holds runs of four channels of one pixel: 8 bytes), then through
    // LDS so that global traffic is 16 bytes per lane
    const int tx = tile % tiles_x, rr = tile / tiles_x, ty = rr % tiles_y, n = rr / tiles_y;
    const int x0 = tx * HT_W, y0 = ty * HT_H;
    bf16_t* ot = reinterpret_cast<bf16_t*>(patch);  // [256 pixels: image row of the patch * 32 + x][OLD]
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int ch = 32 * j + 8 * q4 + 4 * (l >> 5);
        const float4 b4 = *reinterpret_cast<const float4*>(&sbias[ch]);
        const float bv[4] = {b4.x, b4.y, b4.z, b4.w};
#pragma unroll
        for (int i = 0; i < NI; ++i) {
          float v[4];
#pragma unroll
          for (int r = 0; r < 4; ++r) v[r] = fmaxf(acc[i][j][4 * q4 + r] + bv[r], relu_floor);
          uint2 pk;
          pk.x = f2bf_pair(v[0], v[1]);
          pk.y = f2bf_pair(v[2], v[3]);
          *reinterpret_cast<uint2*>(&ot[((NI * w + i) * HT_W + (l & 31)) * OLD + ch]) = pk;
        }
      }
    __syncthreads();
    {
      constexpr int CPR = BN / 8;  // 16-byte chunks per pixel; this thread: chunk t & 7 of pixel column t >> 3, rows 0..7
      const int cc = t & (CPR - 1), px = t >> 3, ox = x0 + px, co = cc * 8;
      const size_t row_step = (size_t)g.Wo * g.Co;
      size_t off = ((size_t)(n * g.Ho + y0) * g.Wo + ox) * g.Co + co;
      if (ox < g.Wo && co < g.Co) {
#pragma unroll
        for (int i = 0; i < HT_H; ++i, off += row_step) {
          if (y0 + i >= g.Ho) break;
          uint4 v = *reinterpret_cast<const uint4*>(&ot[(i * HT_W + px) * OLD + cc * 8]);
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
    }
    if (!has_next) break;
    tile = next_tile;
  }
}

bool g_conv_halo = true;
bool g_conv_halo_resident = true;

}  // namespace

// on: 0 = off, 1 = on, 2 = on but without the weights-resident variant for 64 -> (at most) 64 channels
int set_conv_halo(int on) {
  const int old = !g_conv_halo ? 0 : (g_conv_halo_resident ? 1 : 2);
  if (on >= 0 && on <= 2) {
    g_conv_halo = on != 0;
    g_conv_halo_resident = on == 1;
  }
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
  if (g_conv_halo_resident && g.Ci == HCC && g.Co <= 64) {
    int dev = 0, n_cus = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&n_cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return e;
    const int grid = n_cus >= 8 ? n_cus / 8 * 8 : 8;  // a multiple of 8: the kernel deals tiles out per XCD
    conv3x3_halo_resident_kernel<<<(unsigned)grid, 256, 0, s>>>(x, w, g, ep, tiles_x, tiles_y);
  } else if (g.Co <= 64) {
    conv3x3_halo_kernel<64><<<(unsigned)(g.N * tiles_y * tiles_x), 256, 0, s>>>(x, w, g, ep, tiles_x, tiles_y, 1);
  } else {
    const int tiles_c = (g.Co + 127) / 128;
    conv3x3_halo_kernel<128><<<(unsigned)(g.N * tiles_y * tiles_x * tiles_c), 256, 0, s>>>(x, w, g, ep, tiles_x, tiles_y,
                                                                                           tiles_c);
  }
  return hipGetLastError();
}

}  // namespace pd
