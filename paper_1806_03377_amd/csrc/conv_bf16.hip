// bf16 convolution (NHWC, fp32 accumulate) and max-pooling kernels for gfx950, built on the 32x32x16 MFMA.
//
//   conv_igemm_kernel        implicit GEMM: rows = output pixels, columns = output channels, reduction over
//                            (tap, input channel).  Forward, and dgrad of a stride-1 convolution (the same
//                            kernel on dL/dy with flipped, transposed weights).  Needs Ci % 8 == 0.
//   conv_wgrad_kernel        dW[co][tap][ci] = sum over pixels of dz[p][co] * x[pix(p,tap)][ci]: both operands
//                            are read "sideways" (reduction index = pixel), so 2x8 blocks are transposed on the
//                            way into LDS; the pixel range is split over workgroups, partial sums go to memory
//   wgrad_reduce_update      sums the partials in split order and applies the momentum-SGD update
//   (conv_smallk_bf16.hip)   first layer of an image network (kh*kw*Ci <= 32, e.g. 3x3x3)
//   (conv_wgrad_tr_bf16.hip) weight gradient of stride-1 layers with at most "same" padding
//   maxpool2x2_*             2x2/stride-2 max-pooling; backward sends the gradient to the first maximum in
//                            row-major window order and applies the ReLU mask of the layer below
#include "bf16_util.h"
#include "mfma_util.h"
#include "pd_kernels.h"

namespace pd {
namespace {

__device__ __forceinline__ void store_out(const ConvEpilogue& ep, float v, size_t off, int c) {
  if (ep.bias) v += bf2f(ep.bias[c]);
  if (ep.relu) v = fmaxf(v, 0.f);
  uint16_t o = f2bf(v);
  if (ep.mask && !bf_positive(ep.mask[off])) o = 0;
  ep.out[off] = o;
}

// ------------------------------------------------------------------------------------------------
// implicit-GEMM convolution.  Every wave owns a 64 x 64 block of the output tile (four 32x32 MFMA
// accumulators: two A and two B fragments feed four MFMAs per 16-wide reduction step).  The workgroup's
// four waves are stacked WMW x WNW: 256 pixels x 64 channels for narrow layers, 128 x 128 otherwise.
// grid = (ceil(Co/BN), ceil(N*Ho*Wo/BM)); 64 reduction elements per stage, two stages of loads in flight
// in registers, two LDS buffers.  The finished tile is rounded to bf16, staged in LDS and written out (and
// its ReLU mask read) in 16-byte pieces.  All index arithmetic is 32-bit (the launcher checks the sizes).
// ------------------------------------------------------------------------------------------------
constexpr int CK = 64, CLD = CK + 8, CPD = 2;

template <int WMW, int WNW, bool UP>
__global__ __launch_bounds__(kThreads) void conv_igemm_kernel(const bf16_t* __restrict__ X,
                                                              const bf16_t* __restrict__ Wg, ConvGeom g,
                                                              ConvEpilogue ep) {
  constexpr int BM_ = 64 * WMW, BN_ = 64 * WNW;
  constexpr int ACH = BM_ / 32, BCH = BN_ / 32;  // 16-byte chunks per thread and stage
  constexpr int OLD = BN_ + 8;                   // padded row of the output staging tile (bf16)
  constexpr int kStageElems = (BM_ + BN_) * CLD;
  constexpr int kSmemElems = 2 * kStageElems > BM_ * OLD ? 2 * kStageElems : BM_ * OLD;
  __shared__ __attribute__((aligned(16))) bf16_t smem[kSmemElems];
  bf16_t* const As0 = smem;
  bf16_t* const Bs0 = smem + 2 * BM_ * CLD;
  const int t = threadIdx.x, l = t & 63, w = t >> 6, wm = w / WNW, wn = w % WNW;
  const int co0 = blockIdx.x * BN_;
  const int P = g.N * g.Ho * g.Wo;
  const int p0 = blockIdx.y * BM_;
  const int K = g.kh * g.kw * g.Ci;
  const int T = (K + CK - 1) / CK;
  const int col = t & 7, trow = t >> 3;
  const bool aligned_ci = (g.Ci % CK) == 0;  // then a stage lies inside one tap
  const int per_tap = aligned_ci ? g.Ci / CK : 1;
  // UP: the input is the zero-upsampled tensor; Hl x Wl is its logical size
  const int Hl = UP ? (g.H - 1) * g.up + 1 : g.H, Wl = UP ? (g.W - 1) * g.up + 1 : g.W;

  // the pixel rows this thread loads in every stage
  int hi0[ACH], wi0[ACH], nbase[ACH];
#pragma unroll
  for (int i = 0; i < ACH; ++i) {
    const int p = p0 + trow + 32 * i;
    if (p < P) {
      const unsigned q = (unsigned)p / (unsigned)g.Wo;
      const int wo = p - (int)q * g.Wo;
      const unsigned n = q / (unsigned)g.Ho;
      const int ho = (int)q - (int)n * g.Ho;
      nbase[i] = (int)n * g.H * g.W * g.Ci;
      hi0[i] = ho * g.stride - g.ph;
      wi0[i] = wo * g.stride - g.pw;
    } else {
      nbase[i] = -1;
      hi0[i] = wi0[i] = 0;
    }
  }

  struct Regs {
    uint4 a[ACH], b[BCH];
  };
  auto gload = [&](Regs& r, int st) {
    int tap, ci;
    bool live = st < T;
    if (aligned_ci) {  // wave-uniform decode
      tap = st / per_tap;
      ci = (st - tap * per_tap) * CK + col * 8;
    } else {
      const int k = st * CK + col * 8;
      live = live && k < K;
      tap = live ? k / g.Ci : 0;
      ci = live ? k - tap * g.Ci : 0;
    }
    const int k = tap * g.Ci + ci;
    const int ta = tap / g.kw, tb = tap - ta * g.kw;
#pragma unroll
    for (int i = 0; i < ACH; ++i) {
      int hi = hi0[i] + ta, wi = wi0[i] + tb;
      bool ok = live && nbase[i] >= 0 && (unsigned)hi < (unsigned)Hl && (unsigned)wi < (unsigned)Wl;
      if (UP && ok) {  // only every up-th logical position holds data
        const int hq = hi / g.up, wq = wi / g.up;
        ok = hq * g.up == hi && wq * g.up == wi;
        hi = hq;
        wi = wq;
      }
      r.a[i] = ok ? ldg16(X + (nbase[i] + (hi * g.W + wi) * g.Ci + ci)) : zero16();
    }
#pragma unroll
    for (int i = 0; i < BCH; ++i) {
      const int co = co0 + trow + 32 * i;
      r.b[i] = (live && co < g.Co) ? ldg16(Wg + ((size_t)co * K + k)) : zero16();
    }
  };
  auto sstore = [&](int buf, const Regs& r) {
    bf16_t* as = As0 + buf * BM_ * CLD;
    bf16_t* bs = Bs0 + buf * BN_ * CLD;
#pragma unroll
    for (int i = 0; i < ACH; ++i) *reinterpret_cast<uint4*>(&as[(trow + 32 * i) * CLD + col * 8]) = r.a[i];
#pragma unroll
    for (int i = 0; i < BCH; ++i) *reinterpret_cast<uint4*>(&bs[(trow + 32 * i) * CLD + col * 8]) = r.b[i];
  };

  f32x16 acc[2][2] = {{f32x16{0}, f32x16{0}}, {f32x16{0}, f32x16{0}}};
  Regs Rg[CPD];
#pragma unroll
  for (int p = 0; p < CPD; ++p) gload(Rg[p], p);
  sstore(0, Rg[0]);
  gload(Rg[0], CPD);
  __syncthreads();
  for (int base = 0; base < T; base += CPD) {
#pragma unroll
    for (int j = 0; j < CPD; ++j) {
      const int st = base + j;
      if (st >= T) break;
      const int cur = st & 1;
      const bf16_t* as = As0 + cur * BM_ * CLD;
      const bf16_t* bs = Bs0 + cur * BN_ * CLD;
#pragma unroll
      for (int ks = 0; ks < CK / 16; ++ks) {
        const int kk = ks * 16 + (l >> 5) * 8;
        uint4 a[2], b[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) a[i] = *reinterpret_cast<const uint4*>(&as[(64 * wm + 32 * i + (l & 31)) * CLD + kk]);
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) b[jj] = *reinterpret_cast<const uint4*>(&bs[(64 * wn + 32 * jj + (l & 31)) * CLD + kk]);
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int jj = 0; jj < 2; ++jj)
            acc[i][jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(a[i]), frag(b[jj]), acc[i][jj], 0, 0, 0);
      }
      if (st + 1 < T) {
        sstore(cur ^ 1, Rg[(j + 1) % CPD]);
        gload(Rg[(j + 1) % CPD], st + 1 + CPD);
      }
      __syncthreads();
    }
  }

  if ((g.Co & 7) == 0) {
    // bias / ReLU / rounding in registers, then through LDS so that global traffic is 16 bytes per lane
    bf16_t* ot = smem;  // [BM_][OLD]; all fragment reads are behind the loop's last barrier
#pragma unroll
    for (int jj = 0; jj < 2; ++jj) {
      const int cl = 64 * wn + 32 * jj + (l & 31), c = co0 + cl;
      const float bv = (ep.bias && c < g.Co) ? bf2f(ep.bias[c]) : 0.f;
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float v = acc[i][jj][r] + bv;
          if (ep.relu) v = fmaxf(v, 0.f);
          ot[(64 * wm + 32 * i + 8 * (r >> 2) + 4 * (l >> 5) + (r & 3)) * OLD + cl] = f2bf(v);
        }
    }
    __syncthreads();
    constexpr int CPR = BN_ / 8;  // 16-byte chunks per tile row
#pragma unroll
    for (int i = 0; i < BM_ * CPR / kThreads; ++i) {
      const int c = t + kThreads * i, row = c / CPR, cc = c % CPR;
      const int p = p0 + row, co = co0 + cc * 8;
      if (p >= P || co >= g.Co) continue;
      uint4 v = *reinterpret_cast<const uint4*>(&ot[row * OLD + cc * 8]);
      const size_t off = (size_t)p * g.Co + co;
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
    return;
  }
  // channel counts that are not a multiple of 8 (e.g. dL/dx of a 3-channel input): element-wise stores
#pragma unroll
  for (int jj = 0; jj < 2; ++jj) {
    const int c = co0 + 64 * wn + 32 * jj + (l & 31);
    if (c >= g.Co) continue;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int p = p0 + 64 * wm + 32 * i + 8 * (r >> 2) + 4 * (l >> 5) + (r & 3);
        if (p < P) store_out(ep, acc[i][jj][r], (size_t)p * g.Co + c, c);
      }
  }
}

// ------------------------------------------------------------------------------------------------
// implicit GEMM with direct global -> LDS loads.  256 output pixels x BN output channels per workgroup, four
// waves (BN = 128: 2 x 2 waves of 128 x 64; BN = 64: 4 x 1 waves of 64 x 64), 32 reduction elements per stage,
// three stages in LDS, two workgroups per compute unit (their barriers are independent, so one keeps the matrix
// cores busy while the other waits).  Every lane fetches one 16-byte chunk (8 channels of one tap of one pixel,
// or 8 reduction elements of one filter) per load instruction straight into LDS; the hardware places lane L's
// chunk at M0 + 16 L, i.e. a wave-wide load fills 16 consecutive 64-byte tile rows, and the XOR swizzle of a
// row's four slots is applied by choosing which chunk a lane fetches.  Chunks that fall into the zero padding,
// past the end of the reduction, or beyond the last pixel / channel are fetched from a 16-byte block of zeros, so
// neither padding nor ragged shapes need a second code path.  The loads of stage st+2 are spread between the
// MFMAs of stage st.  (The loads are inline assembly: with the builtin the compiler waits for all outstanding
// loads before every LDS read.)
// ------------------------------------------------------------------------------------------------
__device__ __attribute__((aligned(16))) const uint32_t g_zero16[4] = {0u, 0u, 0u, 0u};
typedef __attribute__((address_space(3))) void lds_void_t;

#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void dma16(const bf16_t* lane_src, char* uniform_lds_dst) {
  const uint32_t lds_addr = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_void_t*)(uniform_lds_dst));
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(lane_src), "s"(lds_addr) : "memory", "m0");
}
#pragma clang diagnostic pop

constexpr int DK = 32, DROWB = DK * 2;

// BN = 64, 128: four waves, three stages, two workgroups per compute unit.  BN = 256 (layers with >= 256 output
// channels): eight waves of 128 x 64 on a 256 x 256 tile, four stages (loads three stages ahead), one workgroup
// per compute unit -- a third fewer operand bytes per MFMA through L2 and LDS than 256 x 128.
template <int BN, bool UP, bool ALIGNED>
__global__ __launch_bounds__(BN == 256 ? 512 : 256, BN == 256 ? 1 : 2) void conv_dma_kernel(const bf16_t* __restrict__ X,
                                                               const bf16_t* __restrict__ Wg, ConvGeom g,
                                                               ConvEpilogue ep) {
  constexpr int BM_ = 256;
  constexpr int NWV = BN == 256 ? 8 : 4, NT_ = 64 * NWV, DNS = BN == 256 ? 4 : 3, D = DNS - 1;
  constexpr int WNW = BN / 64, WMW = NWV / WNW;       // waves along channels / pixels
  constexpr int TM = BM_ / WMW, NI = TM / 32, NJ = 2;  // wave tile TM x 64
  constexpr int QA = 16 / NWV, QB = (BN / 16) / NWV, LPS = QA + QB;   // wave-wide loads per wave and stage
  constexpr int ATILE = BM_ * DROWB, STAGE = (BM_ + BN) * DROWB;
  constexpr int OLD = BN + 8;
  constexpr int kSmem = DNS * STAGE > BM_ * OLD * 2 ? DNS * STAGE : BM_ * OLD * 2;
  constexpr int KS = DK / 16, MF = NI * NJ;
  __shared__ __attribute__((aligned(1024))) char smem[kSmem];
  __shared__ __attribute__((aligned(16))) float sbias[BN];
  const int t = threadIdx.x, l = t & 63;
  const int w = __builtin_amdgcn_readfirstlane(t >> 6), wm = w / WNW, wn = w % WNW;
  // Workgroups are dealt round-robin to the 8 XCDs (each with its own L2): renumber them so that an XCD works on a
  // contiguous run of pixel tiles and the channel tiles of one pixel tile -- they read the same input -- share it.
  int tile_x, tile_y;
  {
    const int ntx = gridDim.x, total = ntx * gridDim.y, per = total >> 3;
    int id = blockIdx.x + ntx * blockIdx.y;
    if (id < per * 8) id = (id & 7) * per + (id >> 3);
    tile_y = id / ntx;
    tile_x = id - tile_y * ntx;
  }
  const int co0 = tile_x * BN;
  const int P = g.N * g.Ho * g.Wo;
  const int p0 = tile_y * BM_;
  // (read in the epilogue, behind every barrier of the pipeline; fetched now so that nobody waits for it there)
  if (t < BN) sbias[t] = (ep.bias && co0 + t < g.Co) ? bf2f(ep.bias[co0 + t]) : 0.f;
  const int K = g.kh * g.kw * g.Ci;
  const int T = (K + DK - 1) / DK;
  const int Hl = UP ? (g.H - 1) * g.up + 1 : g.H, Wl = UP ? (g.W - 1) * g.up + 1 : g.W;
  const bf16_t* const zero = reinterpret_cast<const bf16_t*>(g_zero16);
  const int kg = ((l & 3) ^ ((l >> 4) & 3)) * 8;  // the reduction offset (within a stage) this lane fetches

  constexpr bool FAST = ALIGNED && !UP;  // every stage lies inside one tap and the input is read plainly
  int hi0[QA], wi0[QA], nbase[QA];
  // FAST: per pixel, the element offset of tap (0, 0), channel kg, and one validity bit per tap
  int aoff[QA];
  uint32_t amask[QA];
#pragma unroll
  for (int q = 0; q < QA; ++q) {
    const int p = p0 + (q * NWV + w) * 16 + (l >> 2);
    if (p < P) {
      const unsigned pq = (unsigned)p / (unsigned)g.Wo;
      const int wo = p - (int)pq * g.Wo;
      const unsigned n = pq / (unsigned)g.Ho;
      const int ho = (int)pq - (int)n * g.Ho;
      nbase[q] = (int)n * g.H * g.W * g.Ci;
      hi0[q] = ho * g.stride - g.ph;
      wi0[q] = wo * g.stride - g.pw;
    } else {
      nbase[q] = -1;
      hi0[q] = wi0[q] = 0;
    }
    aoff[q] = nbase[q] + (hi0[q] * g.W + wi0[q]) * g.Ci + kg;
    amask[q] = 0;
    if (FAST && nbase[q] >= 0)
      for (int ta = 0; ta < g.kh; ++ta)
        for (int tb = 0; tb < g.kw; ++tb)
          if ((unsigned)(hi0[q] + ta) < (unsigned)g.H && (unsigned)(wi0[q] + tb) < (unsigned)g.W)
            amask[q] |= 1u << (ta * g.kw + tb);
  }
  int wrow[QB];  // element offset of this lane's filter row, or -1
#pragma unroll
  for (int q = 0; q < QB; ++q) {
    const int co = co0 + (q * NWV + w) * 16 + (l >> 2);
    wrow[q] = co < g.Co ? co * K : -1;
  }
  // FAST: the tap and channel range of the stage being loaded, kept in scalars and advanced once per stage
  int l_kk = 0, l_tap = 0, l_ci = 0, l_ta = 0, l_tb = 0, l_off = 0;
  auto advance_stage = [&]() {
    l_kk += DK;
    l_ci += DK;
    if (l_ci >= g.Ci) {
      l_ci = 0;
      ++l_tap;
      if (++l_tb == g.kw) {
        l_tb = 0;
        ++l_ta;
      }
    }
    l_off = (l_ta * g.W + l_tb) * g.Ci + l_ci;
  };
  // q-th load of the stage whose reduction range starts at kk (A loads first)
  auto load1 = [&](int q, char* stage, int kk) {
    if (FAST) {
      if (q < QA) {
        const bool ok = l_kk < K && ((amask[q] >> l_tap) & 1u);  // past the end of the reduction: zeros
        const bf16_t* cand = X + (aoff[q] + l_off);
        dma16(ok ? cand : zero, stage + (q * NWV + w) * 1024);
      } else {
        const int qb = q - QA;
        const bool ok = l_kk < K && wrow[qb] >= 0;
        const bf16_t* cand = Wg + (wrow[qb] + l_kk + kg);
        dma16(ok ? cand : zero, stage + ATILE + (qb * NWV + w) * 1024);
      }
      return;
    }
    const int k = kk + kg;
    const bf16_t* src = zero;
    if (q < QA) {
      int tap, ci;
      if (ALIGNED) {  // a stage lies inside one tap: wave-uniform decode
        const int tu = kk / g.Ci;
        tap = tu;
        ci = kk - tu * g.Ci + kg;
      } else {
        tap = k / g.Ci;
        ci = k - tap * g.Ci;
      }
      const int ta = tap / g.kw, tb = tap - ta * g.kw;
      int hi = hi0[q] + ta, wi = wi0[q] + tb;
      bool ok = k < K && nbase[q] >= 0 && (unsigned)hi < (unsigned)Hl && (unsigned)wi < (unsigned)Wl;
      if (UP && ok) {
        const int hq = hi / g.up, wq = wi / g.up;
        ok = hq * g.up == hi && wq * g.up == wi;
        hi = hq;
        wi = wq;
      }
      if (ok) src = X + (nbase[q] + (hi * g.W + wi) * g.Ci + ci);
      dma16(src, stage + (q * NWV + w) * 1024);
    } else {
      const int qb = q - QA;
      if (k < K && wrow[qb] >= 0) src = Wg + ((size_t)wrow[qb] + k);
      dma16(src, stage + ATILE + (qb * NWV + w) * 1024);
    }
  };

  f32x16 acc[NI][NJ];
#pragma unroll
  for (int i = 0; i < NI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j) acc[i][j] = f32x16{0};
  int fa[NI], fb[NJ];
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const int row = TM * wm + 32 * i + (l & 31);
    fa[i] = row * DROWB + (((l >> 5) ^ ((row >> 2) & 3)) << 4);
  }
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int row = 64 * wn + 32 * j + (l & 31);
    fb[j] = ATILE + row * DROWB + (((l >> 5) ^ ((row >> 2) & 3)) << 4);
  }
  auto ldf = [&](const char* stage, int o, int ks) { return *reinterpret_cast<const uint4*>(stage + (o ^ (ks << 5))); };

#pragma unroll
  for (int d = 0; d < D; ++d) {
#pragma unroll
    for (int q = 0; q < LPS; ++q) load1(q, smem + d * STAGE, d * DK);
    advance_stage();
  }
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"((D - 1) * LPS) : "memory");  // stage 0 has landed
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  int cur = 0, fill = D;
  for (int st = 0; st < T; ++st) {
    const char* sc = smem + cur * STAGE;
    cur = cur == DNS - 1 ? 0 : cur + 1;
    char* sl = smem + fill * STAGE;
    fill = fill == DNS - 1 ? 0 : fill + 1;
    const int kk = (st + D) * DK;  // past the end of the reduction every chunk comes from the zero block
    uint4 a[2][NI], b[2][NJ];
#pragma unroll
    for (int i = 0; i < NI; ++i) a[0][i] = ldf(sc, fa[i], 0);
#pragma unroll
    for (int j = 0; j < NJ; ++j) b[0][j] = ldf(sc, fb[j], 0);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int c = ks & 1, n = c ^ 1;
      if (ks + 1 < KS) {
#pragma unroll
        for (int i = 0; i < NI; ++i) a[n][i] = ldf(sc, fa[i], ks + 1);
#pragma unroll
        for (int j = 0; j < NJ; ++j) b[n][j] = ldf(sc, fb[j], ks + 1);
      }
      // this k-step's share of the stage's loads: q = ks, ks + KS, ks + 2 KS, ... placed after every other MFMA
#pragma unroll
      for (int m = 0; m < MF; ++m) {
        const int i = m / NJ, j = m % NJ;
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(b[c][j]), frag(a[c][i]), acc[i][j], 0, 0, 0);
        constexpr int kGap = MF >= 8 ? 2 : 1;
        if (m % kGap == kGap - 1) {
          const int q = ks + KS * (m / kGap);
          if (q < LPS) {
            __builtin_amdgcn_sched_barrier(0);
            load1(q, sl, kk);
            __builtin_amdgcn_sched_barrier(0);
          }
        }
      }
    }
    advance_stage();
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"((D - 1) * LPS) : "memory");  // stage st+1 has landed; later ones may be in flight
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();

  // bias / ReLU / rounding in registers, then through LDS so that global traffic is 16 bytes per lane.  The filters
  // are the MFMA's rows, so a lane holds runs of four channels of one pixel: acc[i][j][r] = channel 64 wn + 32 j +
  // 8 (r >> 2) + 4 (l >> 5) + (r & 3) of tile pixel TM wm + 32 i + (l & 31), and a run goes to LDS as 8 bytes.
  bf16_t* ot = reinterpret_cast<bf16_t*>(smem);  // [BM_][OLD]
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
        *reinterpret_cast<uint2*>(&ot[(TM * wm + 32 * i + (l & 31)) * OLD + ch]) = pk;
      }
    }
  __syncthreads();
  constexpr int CPR = BN / 8;
#pragma unroll
  for (int i = 0; i < BM_ * CPR / NT_; ++i) {
    const int c = t + NT_ * i, row = c / CPR, cc = c % CPR;
    const int p = p0 + row, co = co0 + cc * 8;
    if (p >= P || co >= g.Co) continue;
    uint4 v = *reinterpret_cast<const uint4*>(&ot[row * OLD + cc * 8]);
    const size_t off = (size_t)p * g.Co + co;
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

template <int BN>
void launch_dma(hipStream_t s, dim3 grid, const bf16_t* x, const bf16_t* w, const ConvGeom& g, const ConvEpilogue& ep) {
  const bool up = g.up > 1, aligned = (g.Ci % DK) == 0 && g.kh * g.kw <= 32;
  constexpr int threads = BN == 256 ? 512 : 256;
  if (up) {
    if (aligned) conv_dma_kernel<BN, true, true><<<grid, threads, 0, s>>>(x, w, g, ep);
    else conv_dma_kernel<BN, true, false><<<grid, threads, 0, s>>>(x, w, g, ep);
  } else {
    if (aligned) conv_dma_kernel<BN, false, true><<<grid, threads, 0, s>>>(x, w, g, ep);
    else conv_dma_kernel<BN, false, false><<<grid, threads, 0, s>>>(x, w, g, ep);
  }
}

bool g_conv_dma = true;
int g_conv_wide_min_tiles = 256;  // 256 x 256 output tiles from which the wide kernel is used (one per compute unit)

hipError_t launch_igemm(hipStream_t s, const bf16_t* x, const bf16_t* w, const ConvGeom& g, const ConvEpilogue& ep) {
  const long long P = (long long)g.N * g.Ho * g.Wo;
  if ((long long)g.N * g.H * g.W * g.Ci >= (1ll << 31) || P * g.Co >= (1ll << 31) || (g.Ci % 8))
    return hipErrorInvalidValue;
  if (conv3x3_halo_applies(g, x, w)) return conv3x3_halo_bf16(s, x, w, g, ep);
  if (g_conv_dma && (g.Co % 8) == 0 && (long long)g.Co * g.kh * g.kw * g.Ci < (1ll << 31) &&
      ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(w)) & 15) == 0) {
    // 256-wide tiles only when they fill the chip about as well as 128-wide ones would: a launch of n equal tiles
    // keeps the 256 compute units busy for n / (256 ceil(n / 256)) of its time, and the wide tile is worth about a
    // tenth more per tile (56 x 56 x 256 layers at minibatch 64: 784 wide tiles = 3.06 rounds against 1568 narrow
    // ones = 6.1 rounds; measured 2 % of the whole convolution stage in favour of the narrow tiles)
    const long long tiles256 = ((g.Co + 255) / 256) * ((P + 255) / 256);
    const long long tiles128 = ((g.Co + 127) / 128) * ((P + 255) / 256);
    auto fill = [](long long n) { return (double)n / (double)(((n + 255) / 256) * 256); };
    const long long tiles64 = ((g.Co + 63) / 64) * ((P + 255) / 256);
    if (g.Co <= 64) launch_dma<64>(s, dim3(1, (unsigned)((P + 255) / 256)), x, w, g, ep);
    // fewer 128-wide tiles than compute units: more, narrower ones (the 17 x 17 layers of the Inception-shaped network at
    // minibatch 64 have 73 pixel tiles; that pipeline 10.49 -> 10.26 ms per minibatch)
    else if (tiles128 < 256 && tiles64 > tiles128)
      launch_dma<64>(s, dim3((g.Co + 63) / 64, (unsigned)((P + 255) / 256)), x, w, g, ep);
    else if (g.Co >= 256 && (g.Co % 256 == 0 || g.Co > 512) && tiles256 >= g_conv_wide_min_tiles &&
             1.1 * fill(tiles256) >= fill(tiles128))
      launch_dma<256>(s, dim3((g.Co + 255) / 256, (unsigned)((P + 255) / 256)), x, w, g, ep);
    else launch_dma<128>(s, dim3((g.Co + 127) / 128, (unsigned)((P + 255) / 256)), x, w, g, ep);
    return hipGetLastError();
  }
  const bool up = g.up > 1;
  if (g.Co <= 64) {
    dim3 grid(1, (unsigned)((P + 255) / 256));
    if (up) conv_igemm_kernel<4, 1, true><<<grid, kThreads, 0, s>>>(x, w, g, ep);
    else conv_igemm_kernel<4, 1, false><<<grid, kThreads, 0, s>>>(x, w, g, ep);
  } else {
    dim3 grid((g.Co + 127) / 128, (unsigned)((P + 127) / 128));
    if (up) conv_igemm_kernel<2, 2, true><<<grid, kThreads, 0, s>>>(x, w, g, ep);
    else conv_igemm_kernel<2, 2, false><<<grid, kThreads, 0, s>>>(x, w, g, ep);
  }
  return hipGetLastError();
}

// wt[ci][kh-1-a][kw-1-b][co] = w[co][a][b][ci]: the weights of the stride-1 convolution that maps dL/dy to dL/dx
__global__ __launch_bounds__(256) void flip_transpose_kernel(const bf16_t* __restrict__ w, bf16_t* __restrict__ wt,
                                                             int Co, int kh, int kw, int Ci) {
  const size_t n = (size_t)Co * kh * kw * Ci;
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n) return;
  const int ci = (int)(idx % Ci);
  size_t q = idx / Ci;
  const int b = (int)(q % kw);
  q /= kw;
  const int a = (int)(q % kh);
  const int co = (int)(q / kh);
  wt[(((size_t)ci * kh + (kh - 1 - a)) * kw + (kw - 1 - b)) * Co + co] = w[idx];
}

// ------------------------------------------------------------------------------------------------
// weight gradient, partial over a pixel range.
// grid.x = co-tiles * ci-tiles * taps (tap fastest), grid.y = splits.  Tile TC x TC of (co, ci) for one tap.
// part[split][e], e = (co*taps + tap)*Ci + ci for the weights, n_w + co for the bias (column sums of dz,
// written by the workgroups of tap 0, ci-tile 0).
// ------------------------------------------------------------------------------------------------
template <int TC>
__global__ __launch_bounds__(kThreads) void conv_wgrad_kernel(const bf16_t* __restrict__ dZ,
                                                              const bf16_t* __restrict__ X, float* __restrict__ part,
                                                              ConvGeom g, int chunks_per_split) {
  constexpr int NBLK = TC / 8 * 32 / kThreads;  // 2x8 blocks per thread and operand (1 for 64, 2 for 128)
  constexpr int WB = TC / 64;                   // 32x32 blocks per wave along each side
  __shared__ __attribute__((aligned(16))) uint32_t Zt[2][TC * 32];  // [co][64 pixels], swizzled
  __shared__ __attribute__((aligned(16))) uint32_t Xt[2][TC * 32];  // [ci][64 pixels]
  const int t = threadIdx.x, l = t & 63, w = t >> 6, wr = w >> 1, wc = w & 1;
  const int taps = g.kh * g.kw;
  const int ci_tiles = (g.Ci + TC - 1) / TC;
  const int tap = blockIdx.x % taps;
  const int ci0 = ((blockIdx.x / taps) % ci_tiles) * TC;
  const int co0 = (blockIdx.x / taps / ci_tiles) * TC;
  const int ta = tap / g.kw, tb = tap - ta * g.kw;
  const long long P = (long long)g.N * g.Ho * g.Wo;
  const long long chunk0 = (long long)blockIdx.y * chunks_per_split;
  const long long nchunks_total = (P + 63) / 64;
  long long chunk1 = chunk0 + chunks_per_split;
  if (chunk1 > nchunks_total) chunk1 = nchunks_total;
  const bool do_bias = tap == 0 && ci0 == 0;

  struct Regs {
    uint4 z0[NBLK], z1[NBLK], x0[NBLK], x1[NBLK];
  };
  auto gload = [&](Regs& r, long long ch) {
    const bool live = ch < chunk1;
#pragma unroll
    for (int i = 0; i < NBLK; ++i) {
      const int b = t + kThreads * i, cc = b % (TC / 8), pair = b / (TC / 8);
      const long long p = ch * 64 + 2 * pair;
      const int co = co0 + 8 * cc, ci = ci0 + 8 * cc;
      r.z0[i] = (live && p < P && co < g.Co) ? ldg16(dZ + (size_t)p * g.Co + co) : zero16();
      r.z1[i] = (live && p + 1 < P && co < g.Co) ? ldg16(dZ + (size_t)(p + 1) * g.Co + co) : zero16();
      uint4 xv[2];
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const long long pp = p + h;
        bool ok = live && pp < P && ci < g.Ci;
        long long off = 0;
        if (ok) {
          const int wo = (int)(pp % g.Wo);
          const long long q = pp / g.Wo;
          const int ho = (int)(q % g.Ho);
          const int hi = ho * g.stride - g.ph + ta, wi = wo * g.stride - g.pw + tb;
          ok = hi >= 0 && hi < g.H && wi >= 0 && wi < g.W;
          off = (((q / g.Ho) * g.H + hi) * (long long)g.W + wi) * g.Ci + ci;
        }
        xv[h] = ok ? ldg16(X + off) : zero16();
      }
      r.x0[i] = xv[0];
      r.x1[i] = xv[1];
    }
  };
  auto sstore = [&](int buf, const Regs& r) {
#pragma unroll
    for (int i = 0; i < NBLK; ++i) {
      const int b = t + kThreads * i, cc = b % (TC / 8), pair = b / (TC / 8);
      store_transposed_pair<8>(Zt[buf], 8 * cc, pair, r.z0[i], r.z1[i]);
      store_transposed_pair<8>(Xt[buf], 8 * cc, pair, r.x0[i], r.x1[i]);
    }
  };

  f32x16 acc[WB][WB];
#pragma unroll
  for (int i = 0; i < WB; ++i)
#pragma unroll
    for (int j = 0; j < WB; ++j) acc[i][j] = f32x16{0};
  float bsum = 0.f;

  if (chunk0 < chunk1) {
    Regs R;
    gload(R, chunk0);
    sstore(0, R);
    __syncthreads();
    for (long long ch = chunk0; ch < chunk1; ++ch) {
      const int cur = (int)((ch - chunk0) & 1);
      gload(R, ch + 1);
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const int grp = 2 * ks + (l >> 5);
        uint4 a[WB], b[WB];
#pragma unroll
        for (int i = 0; i < WB; ++i) a[i] = load_swizzled_frag<8>(Zt[cur], 32 * (WB * wr + i) + (l & 31), grp);
#pragma unroll
        for (int j = 0; j < WB; ++j) b[j] = load_swizzled_frag<8>(Xt[cur], 32 * (WB * wc + j) + (l & 31), grp);
#pragma unroll
        for (int i = 0; i < WB; ++i)
#pragma unroll
          for (int j = 0; j < WB; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(a[i]), frag(b[j]), acc[i][j], 0, 0, 0);
      }
      if (do_bias && t < TC) {  // this channel's 64 dz values of the chunk, in pixel order
#pragma unroll
        for (int grp = 0; grp < 8; ++grp) {
          const uint4 v = load_swizzled_frag<8>(Zt[cur], t, grp);
          const uint32_t ww[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            bsum += bf2f((uint16_t)(ww[q] & 0xffffu));
            bsum += bf2f((uint16_t)(ww[q] >> 16));
          }
        }
      }
      if (ch + 1 < chunk1) sstore(cur ^ 1, R);
      __syncthreads();
    }
  }

  const size_t n_w = (size_t)g.Co * taps * g.Ci;
  float* out = part + (size_t)blockIdx.y * (n_w + g.Co);
#pragma unroll
  for (int j = 0; j < WB; ++j) {
    const int ci = ci0 + 32 * (WB * wc + j) + (l & 31);
    if (ci >= g.Ci) continue;
#pragma unroll
    for (int i = 0; i < WB; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int co = co0 + 32 * (WB * wr + i) + 8 * (r >> 2) + 4 * (l >> 5) + (r & 3);
        if (co < g.Co) out[((size_t)co * taps + tap) * g.Ci + ci] = acc[i][j][r];
      }
  }
  if (do_bias && t < TC && co0 + t < g.Co) out[n_w + co0 + t] = bsum;
}

// g[e] = sum over splits of part[s][e]; then m <- mu*m + g; w <- w - lr*m; ring <- bf16(w).
// e < n_w addresses the weights, e >= n_w the bias.  G adjacent lanes share one element: lane j adds the splits
// j, j + G, j + 2G, ... in that order, then the G sums are combined pairwise (a fixed tree), so the result depends
// only on (splits, G).  G = 1 is the plain sequential sum; larger G keeps the chip busy when a layer has few
// parameters but many partial sums.
template <int G>
__global__ __launch_bounds__(256) void wgrad_reduce_update_kernel(const float* __restrict__ part, int splits,
                                                                  size_t stride, size_t n_w, int n_b, float* __restrict__ master_w,
                                                                  float* __restrict__ mom_w, bf16_t* __restrict__ ring_w,
                                                                  float* __restrict__ master_b, float* __restrict__ mom_b,
                                                                  bf16_t* __restrict__ ring_b, UpdateRule rule) {
  const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t e = tid / G;
  const int j = (int)(tid % G);
  const size_t n = n_w + n_b;
  const bool live = e < n;  // (whole groups of G lanes are live or not: 256 % G == 0)
  float gsum = 0.f;
  if (live)
    for (int s = j; s < splits; s += G) gsum += part[(size_t)s * stride + e];
#pragma unroll
  for (int d = 1; d < G; d <<= 1) gsum += __shfl_xor(gsum, d, 64);
  if (!live || j != 0) return;
  float* ms = e < n_w ? master_w + e : master_b + (e - n_w);
  float* mm = e < n_w ? mom_w + e : mom_b + (e - n_w);
  bf16_t* rr = e < n_w ? ring_w + e : ring_b + (e - n_w);
  if (rule.kind == kRuleGradOnly) {  // replicated stage: the sum over replicas comes first
    *ms = gsum;
    return;
  }
  float m = *mm, wv = *ms;
  apply_update(rule, gsum, m, wv);
  *mm = m;
  *ms = wv;
  *rr = f2bf(wv);
}

// ------------------------------------------------------------------------------------------------
// 2x2 / stride-2 max pooling over NHWC, 8 channels (16 bytes) per thread.
// ------------------------------------------------------------------------------------------------
// route (optional): one 32-bit word per thread, four bits per channel: bits 0-1 = the window position (2 a + b) of
// the first maximum, bit 2 = that maximum is positive, bit 3 = it is not a NaN.  The backward pass needs nothing else
// of x and y: it reads the gradient and these words (an eighth of y's bytes) instead of x, y and the gradient.
__global__ __launch_bounds__(256) void maxpool2x2_fwd_kernel(const bf16_t* __restrict__ x, bf16_t* __restrict__ y,
                                                             uint32_t* __restrict__ route, int N, int H, int W, int C) {
  const int Ho = H / 2, Wo = W / 2, C8 = C / 8;
  const size_t total = (size_t)N * Ho * Wo * C8;
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int c8 = (int)(idx % C8);
  size_t q = idx / C8;
  const int wo = (int)(q % Wo);
  q /= Wo;
  const int ho = (int)(q % Ho);
  const size_t n = q / Ho;
  float best[8];
  uint16_t bo[8];
  uint32_t pos[8];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      uint16_t v[8];
      unpack8(ldg16(x + ((n * H + 2 * ho + a) * W + 2 * wo + b) * C + 8 * c8), v);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float f = bf2f(v[j]);
        if ((a == 0 && b == 0) || f > best[j]) {
          best[j] = f;
          bo[j] = v[j];
          pos[j] = (uint32_t)(2 * a + b);
        }
      }
    }
  *reinterpret_cast<uint4*>(y + ((n * Ho + ho) * Wo + wo) * C + 8 * c8) = pack8(bo);
  if (route) {
    uint32_t r = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j)
      r |= (pos[j] | (bf_positive(bo[j]) ? 4u : 0u) | (best[j] == best[j] ? 8u : 0u)) << (4 * j);
    route[idx] = r;
  }
}

// The backward pass from the routing words alone: dx[window position] = dy where the position is the recorded one and
// the maximum was not a NaN (a NaN equals nothing, so the comparing kernel below routes nothing either) and, with
// relu_mask, was positive (x at that position IS the maximum); 0 elsewhere.
__global__ __launch_bounds__(256) void maxpool2x2_bwd_route_kernel(const uint32_t* __restrict__ route,
                                                                   const bf16_t* __restrict__ dy, bf16_t* __restrict__ dx,
                                                                   int N, int H, int W, int C, int relu_mask) {
  const int Ho = H / 2, Wo = W / 2, C8 = C / 8;
  const size_t total = (size_t)N * Ho * Wo * C8;
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int c8 = (int)(idx % C8);
  size_t q = idx / C8;
  const int wo = (int)(q % Wo);
  q /= Wo;
  const int ho = (int)(q % Ho);
  const size_t n = q / Ho;
  uint16_t dv[8];
  unpack8(ldg16(dy + ((n * Ho + ho) * Wo + wo) * C + 8 * c8), dv);
  const uint32_t r = route[idx];
  const uint32_t need = relu_mask ? 12u : 8u;
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      uint16_t o[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const uint32_t code = (r >> (4 * j)) & 15u;
        o[j] = ((code & 3u) == (uint32_t)(2 * a + b) && (code & need) == need) ? dv[j] : (uint16_t)0;
      }
      *reinterpret_cast<uint4*>(dx + ((n * H + 2 * ho + a) * W + 2 * wo + b) * C + 8 * c8) = pack8(o);
    }
}

// dx[window] = dy at the first position whose value equals the window maximum, else 0; with relu_mask also 0
// where x <= 0 (the ReLU of the layer that produced x).
__global__ __launch_bounds__(256) void maxpool2x2_bwd_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ y,
                                                             const bf16_t* __restrict__ dy, bf16_t* __restrict__ dx,
                                                             int N, int H, int W, int C, int relu_mask) {
  const int Ho = H / 2, Wo = W / 2, C8 = C / 8;
  const size_t total = (size_t)N * Ho * Wo * C8;
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int c8 = (int)(idx % C8);
  size_t q = idx / C8;
  const int wo = (int)(q % Wo);
  q /= Wo;
  const int ho = (int)(q % Ho);
  const size_t n = q / Ho;
  uint16_t yv[8], dv[8];
  const size_t yoff = ((n * Ho + ho) * Wo + wo) * C + 8 * c8;
  unpack8(ldg16(y + yoff), yv);
  unpack8(ldg16(dy + yoff), dv);
  bool taken[8] = {false, false, false, false, false, false, false, false};
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      const size_t xoff = ((n * H + 2 * ho + a) * W + 2 * wo + b) * C + 8 * c8;
      uint16_t xv[8], o[8];
      unpack8(ldg16(x + xoff), xv);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const bool hit = !taken[j] && bf2f(xv[j]) == bf2f(yv[j]);
        taken[j] = taken[j] || hit;
        o[j] = (hit && (!relu_mask || bf_positive(xv[j]))) ? dv[j] : (uint16_t)0;
      }
      *reinterpret_cast<uint4*>(dx + xoff) = pack8(o);
    }
}

int wgrad_splits(long long chunks, int tiles) {
  long long s = 3072 / (tiles > 0 ? tiles : 1);
  if (s > chunks / 16) s = chunks / 16;
  if (s > 1024) s = 1024;
  if (s < 1) s = 1;
  return (int)s;
}

}  // namespace


void set_conv_wide_min_tiles(int min_tiles) {
  if (min_tiles >= 1) g_conv_wide_min_tiles = min_tiles;
}

int conv_wgrad_split_count(const ConvGeom& g) {
  const long long P = (long long)g.N * g.Ho * g.Wo;
  if (conv_is_smallk(g)) return wgrad_splits((P + 255) / 256, 1);
  if (const int tr = conv_wgrad_tr_partials(g)) return tr;
  const int TC = (g.Co >= 128 && g.Ci >= 128) ? 128 : 64;
  const int tiles = ((g.Co + TC - 1) / TC) * ((g.Ci + TC - 1) / TC) * g.kh * g.kw;
  return wgrad_splits((P + 63) / 64, tiles);
}

hipError_t conv_forward_bf16(hipStream_t s, const bf16_t* x, const bf16_t* w, const ConvGeom& g,
                             const ConvEpilogue& ep) {
  const long long P = (long long)g.N * g.Ho * g.Wo;
  (void)P;
  if (conv_is_smallk(g)) return conv_smallk_forward_bf16(s, x, w, g, ep);
  return launch_igemm(s, x, w, g, ep);
}

hipError_t conv_dgrad_bf16(hipStream_t s, const bf16_t* dz, const bf16_t* w, bf16_t* wt_scratch, const ConvGeom& g,
                           const ConvEpilogue& ep) {
  if (g.stride < 1 || (g.Co % 8)) return hipErrorInvalidValue;
  const size_t n = (size_t)g.Co * g.kh * g.kw * g.Ci;
  flip_transpose_kernel<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(w, wt_scratch, g.Co, g.kh, g.kw, g.Ci);
  // the transposed convolution: dL/dy [N][Ho][Wo][Co] (zero-upsampled by the stride) -> dL/dx [N][H][W][Ci], a
  // stride-1 convolution with the flipped weights and padding k-1-p; input rows/columns the forward pass never
  // touched (when (H + 2p - k) % stride != 0) fall outside the upsampled tensor and come out as zero
  ConvGeom t = g;
  t.H = g.Ho; t.W = g.Wo; t.Ci = g.Co; t.Ho = g.H; t.Wo = g.W; t.Co = g.Ci;
  t.ph = g.kh - 1 - g.ph; t.pw = g.kw - 1 - g.pw;
  t.stride = 1; t.up = g.stride;
  return launch_igemm(s, dz, wt_scratch, t, ep);
}

hipError_t conv_wgrad_partial_bf16(hipStream_t s, const bf16_t* dz, const bf16_t* x, float* part, int splits,
                                   const ConvGeom& g) {
  const long long P = (long long)g.N * g.Ho * g.Wo;
  if (conv_is_smallk(g)) return conv_smallk_wgrad_partial_bf16(s, dz, x, part, splits, g);
  if ((g.Ci % 8) || (g.Co % 8)) return hipErrorInvalidValue;
  if (conv_wgrad_tr_partials(g)) return conv_wgrad_tr_partial_bf16(s, dz, x, part, splits, g);
  const long long chunks = (P + 63) / 64;
  const int cps = (int)((chunks + splits - 1) / splits);
  if (g.Co >= 128 && g.Ci >= 128) {
    dim3 grid(((g.Co + 127) / 128) * ((g.Ci + 127) / 128) * g.kh * g.kw, splits);
    conv_wgrad_kernel<128><<<grid, kThreads, 0, s>>>(dz, x, part, g, cps);
  } else {
    dim3 grid(((g.Co + 63) / 64) * ((g.Ci + 63) / 64) * g.kh * g.kw, splits);
    conv_wgrad_kernel<64><<<grid, kThreads, 0, s>>>(dz, x, part, g, cps);
  }
  return hipGetLastError();
}

// The same four elements at a time (16-byte accesses; a group of four never straddles the weight / bias border
// because both counts are multiples of four).  Lane j of a group adds the splits j, j + G, ... in that order, as
// above, but their loads are issued in batches of eight before the first add (unconditional loads of a clamped
// split index, surplus terms dropped by a select), and master and momentum are requested right after the first
// batch: the kernel is a chain of memory latencies otherwise (one 4-byte load per add, then two more loads).
template <int G>
__global__ __launch_bounds__(256) void wgrad_reduce_update4_kernel(const float* __restrict__ part, int splits,
                                                                   size_t stride, size_t n_w, int n_b,
                                                                   float* __restrict__ master_w, float* __restrict__ mom_w,
                                                                   bf16_t* __restrict__ ring_w, float* __restrict__ master_b,
                                                                   float* __restrict__ mom_b, bf16_t* __restrict__ ring_b,
                                                                   UpdateRule rule) {
  constexpr int kBatch = 8;
  const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t e = (tid / G) * 4;
  const int j = (int)(tid % G);
  const size_t n = n_w + n_b;
  const bool live = e < n;  // (whole groups of G lanes are live or not: 256 % G == 0)
  const size_t ec = live ? e : 0;
  const bool is_w = ec < n_w;
  float* ms = is_w ? master_w + ec : master_b + (ec - n_w);
  float* mm = is_w ? mom_w + ec : mom_b + (ec - n_w);
  bf16_t* rr = is_w ? ring_w + ec : ring_b + (ec - n_w);
  const int terms = (splits + G - 1) / G;  // per lane, counting the ones past the end that are dropped
  float4 g = make_float4(0.f, 0.f, 0.f, 0.f), m4 = g, w4 = g;
  for (int i0 = 0; i0 < terms; i0 += kBatch) {
    float4 p[kBatch];
#pragma unroll
    for (int q = 0; q < kBatch; ++q) {
      const int sx = j + (i0 + q) * G;
      p[q] = *reinterpret_cast<const float4*>(part + (size_t)(sx < splits ? sx : j) * stride + ec);
    }
    if (i0 == 0 && rule.kind != kRuleGradOnly) {
      m4 = *reinterpret_cast<const float4*>(mm);
      w4 = *reinterpret_cast<const float4*>(ms);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int q = 0; q < kBatch; ++q) {
      const bool on = j + (i0 + q) * G < splits;
      g.x = on ? g.x + p[q].x : g.x; g.y = on ? g.y + p[q].y : g.y;
      g.z = on ? g.z + p[q].z : g.z; g.w = on ? g.w + p[q].w : g.w;
    }
  }
#pragma unroll
  for (int d = 1; d < G; d <<= 1) {
    g.x += __shfl_xor(g.x, d, 64); g.y += __shfl_xor(g.y, d, 64);
    g.z += __shfl_xor(g.z, d, 64); g.w += __shfl_xor(g.w, d, 64);
  }
  if (!live || j != 0) return;
  if (rule.kind == kRuleGradOnly) {  // replicated stage: the sum over replicas comes first
    *reinterpret_cast<float4*>(ms) = g;
    return;
  }
  apply_update(rule, g.x, m4.x, w4.x); apply_update(rule, g.y, m4.y, w4.y);
  apply_update(rule, g.z, m4.z, w4.z); apply_update(rule, g.w, m4.w, w4.w);
  *reinterpret_cast<float4*>(mm) = m4;
  *reinterpret_cast<float4*>(ms) = w4;
  uint2 pk;
  pk.x = (uint32_t)f2bf(w4.x) | ((uint32_t)f2bf(w4.y) << 16);
  pk.y = (uint32_t)f2bf(w4.z) | ((uint32_t)f2bf(w4.w) << 16);
  *reinterpret_cast<uint2*>(rr) = pk;
}

hipError_t wgrad_reduce_update(hipStream_t s, const float* part, int splits, size_t stride, size_t n_w, int n_b,
                               float* master_w, float* mom_w, bf16_t* ring_w, float* master_b, float* mom_b,
                               bf16_t* ring_b, UpdateRule rule) {
  const size_t n = n_w + n_b;
  if (!stride) stride = n;
  const uintptr_t align16 = reinterpret_cast<uintptr_t>(part) | reinterpret_cast<uintptr_t>(master_w) |
                            reinterpret_cast<uintptr_t>(mom_w) | reinterpret_cast<uintptr_t>(master_b) |
                            reinterpret_cast<uintptr_t>(mom_b);
  const uintptr_t align8 = reinterpret_cast<uintptr_t>(ring_w) | reinterpret_cast<uintptr_t>(ring_b);
  if (splits >= 1 && (n_w % 4) == 0 && (n_b % 4) == 0 && (stride % 4) == 0 && (align16 & 15) == 0 && (align8 & 7) == 0) {
    int G = 1;
    while (G < 64 && 2 * G <= splits && (n / 4) * (size_t)(2 * G) <= ((size_t)1 << 19)) G *= 2;
    const unsigned blocks = (unsigned)((n / 4 * G + 255) / 256);
#define PD_REDUCE4(GG)                                                                                              \
  wgrad_reduce_update4_kernel<GG><<<blocks, 256, 0, s>>>(part, splits, stride, n_w, n_b, master_w, mom_w, ring_w, \
                                                         master_b, mom_b, ring_b, rule)
    switch (G) {
      case 1: PD_REDUCE4(1); break;
      case 2: PD_REDUCE4(2); break;
      case 4: PD_REDUCE4(4); break;
      case 8: PD_REDUCE4(8); break;
      case 16: PD_REDUCE4(16); break;
      case 32: PD_REDUCE4(32); break;
      default: PD_REDUCE4(64); break;
    }
#undef PD_REDUCE4
    return hipGetLastError();
  }
  // lanes per element: enough threads to fill the chip, never more than there are partial sums
  int G = 1;
  while (G < 64 && 2 * G <= splits && n * (size_t)(2 * G) <= ((size_t)1 << 19)) G *= 2;
  const unsigned blocks = (unsigned)((n * G + 255) / 256);
#define PD_REDUCE(GG)                                                                                              \
  wgrad_reduce_update_kernel<GG><<<blocks, 256, 0, s>>>(part, splits, stride, n_w, n_b, master_w, mom_w, ring_w, \
                                                        master_b, mom_b, ring_b, rule)
  switch (G) {
    case 1: PD_REDUCE(1); break;
    case 2: PD_REDUCE(2); break;
    case 4: PD_REDUCE(4); break;
    case 8: PD_REDUCE(8); break;
    case 16: PD_REDUCE(16); break;
    case 32: PD_REDUCE(32); break;
    default: PD_REDUCE(64); break;
  }
#undef PD_REDUCE
  return hipGetLastError();
}

hipError_t maxpool2x2_forward_bf16(hipStream_t s, const bf16_t* x, bf16_t* y, uint32_t* route, int N, int H, int W,
                                   int C) {
  if ((C % 8) || (H % 2) || (W % 2)) return hipErrorInvalidValue;
  const size_t total = (size_t)N * (H / 2) * (W / 2) * (C / 8);
  maxpool2x2_fwd_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>(x, y, route, N, H, W, C);
  return hipGetLastError();
}

hipError_t maxpool2x2_backward_routed_bf16(hipStream_t s, const uint32_t* route, const bf16_t* dy, bf16_t* dx, int N,
                                           int H, int W, int C, bool relu_mask) {
  if ((C % 8) || (H % 2) || (W % 2)) return hipErrorInvalidValue;
  const size_t total = (size_t)N * (H / 2) * (W / 2) * (C / 8);
  maxpool2x2_bwd_route_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>(route, dy, dx, N, H, W, C,
                                                                              relu_mask ? 1 : 0);
  return hipGetLastError();
}

hipError_t maxpool2x2_backward_bf16(hipStream_t s, const bf16_t* x, const bf16_t* y, const bf16_t* dy, bf16_t* dx, int N,
                                    int H, int W, int C, bool relu_mask) {
  if ((C % 8) || (H % 2) || (W % 2)) return hipErrorInvalidValue;
  const size_t total = (size_t)N * (H / 2) * (W / 2) * (C / 8);
  maxpool2x2_bwd_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>(x, y, dy, dx, N, H, W, C, relu_mask ? 1 : 0);
  return hipGetLastError();
}

}  // namespace pd
