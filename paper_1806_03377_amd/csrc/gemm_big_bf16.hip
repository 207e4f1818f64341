// Compute-bound bf16 GEMM for gfx950: 256 x 256 output tile per workgroup, 128 x 128 per wave (sixteen 32x32
// MFMA accumulators = 256 accumulation registers), 64 reduction elements per stage.
//
//   out[I][J] = sum_r A(i,r) * B(r,j)
//     TA = false: A is stored [I][R] (reduction contiguous)     TA = true: A is stored [R][I]
//     TB = false: B is stored [J][R] (reduction contiguous)     TB = true: B is stored [R][J]
//   forward  y  = x w^T      : A = x  (TA=0), B = w (TB=0), I = rows, J = out-features, R = in-features
//   dgrad    dx = dz w       : A = dz (TA=0), B = w (TB=1), I = rows, J = in-features,  R = out-features
//   wgrad    dW = dz^T x     : A = dz (TA=1), B = x (TB=1), I = out-features, J = in-features, R = rows
//
// Why this shape: with one wave per SIMD, a wave tile of m x n reads (m + n) * 32 bytes of fragments from LDS
// per sixteen-wide reduction step and issues (m/32)(n/32) MFMAs of 32 cycles; four waves at 64 x 64 already ask
// for the whole LDS read bandwidth, at 128 x 128 for half of it.  Operands stored "sideways" are transposed in
// 2x8 blocks on their way into a swizzled LDS tile, so every fragment read is a 16-byte access.
#include "bf16_util.h"
#include "mfma_util.h"
#include "pd_kernels.h"

namespace pd {
namespace {

constexpr int GM = 256, GN = 256, GK = 64, GLD = GK + 8;

struct BigEpilogue {
  const bf16_t* bias;  // [J] or null
  const bf16_t* mask;  // [I][J] (> 0 keeps) or null
  int relu;
  bf16_t* out;         // [I][J] bf16, or
  float* out_f;        // [I][J] fp32 (no rounding; bias/ReLU still applied)
  int ldo;             // row stride of out / out_f / mask (elements)
  // Momentum-SGD step fused into the store (weight gradients): the result g is not written; instead
  // m <- mu*m + g; w <- w - lr*m; ring <- bf16(w) on [I][J] arrays with row stride ldo.  Null: off.
  float* upd_master;
  float* upd_mom;
  bf16_t* upd_ring;
  UpdateRule rule;
};

// Epilogue of one wave's 128 x WCOLS sub-tile (accumulators acc[4][NJ], top-left corner row0, col_base): bias,
// ReLU, rounding, mask.  The wave stages 32-row blocks in its private LDS region `stage` (the operand tiles are
// dead by then) and writes them out as full rows, 16 bytes per lane.
// (NJT = column blocks the wave holds, of which this call handles NJ starting at block J0: a wave with 128 columns
// goes through two calls of 64, which keeps the fully unrolled body at the size the compiler still unrolls -- with
// anything less the accumulators are indexed dynamically and end up in scratch memory.)
template <int NJ, int WCOLS, int NJT = NJ, int J0 = 0>
__device__ __forceinline__ void big_epilogue(f32x16 (&acc_all)[4][NJT], const BigEpilogue& ep, char* stage, int row0,
                                             int col_base, int l, int I, int J) {
  auto acc = [&](int i, int j) -> f32x16& { return acc_all[i][J0 + j]; };
  const bool wide_ok = ((ep.ldo & 7) == 0) && ((J & 7) == 0);
  if (wide_ok) {
    constexpr int FLD = WCOLS + 4, HLD = WCOLS + 8;  // padded staging rows (fp32 / bf16)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row_base = row0 + 32 * i;
      if (ep.out_f || ep.upd_master) {
        float* sf = reinterpret_cast<float*>(stage);  // [32][FLD]
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
          const int c = col_base + 32 * j + (l & 31);
          const float bv = (ep.bias && c < J) ? bf2f(ep.bias[c]) : 0.f;
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            float v = acc(i, j)[r] + bv;
            if (ep.relu) v = fmaxf(v, 0.f);
            sf[(8 * (r >> 2) + 4 * (l >> 5) + (r & 3)) * FLD + 32 * j + (l & 31)] = v;
          }
        }
        constexpr int LPR = WCOLS / 4;       // lanes per row (float4 each)
        constexpr int RPP = 64 / LPR;        // rows per pass
#pragma unroll
        for (int q = 0; q < 32 / RPP; ++q) {
          const int rr = RPP * q + l / LPR, cc = (l % LPR) * 4;
          const int row = row_base + rr, c = col_base + cc;
          if (row < I && c < J) {
            const float4 v = *reinterpret_cast<const float4*>(&sf[rr * FLD + cc]);
            const size_t off = (size_t)row * ep.ldo + c;
            if (ep.upd_master) {
              float4 mm = *reinterpret_cast<const float4*>(ep.upd_mom + off);
              float4 ms = *reinterpret_cast<const float4*>(ep.upd_master + off);
              apply_update(ep.rule, v.x, mm.x, ms.x); apply_update(ep.rule, v.y, mm.y, ms.y);
              apply_update(ep.rule, v.z, mm.z, ms.z); apply_update(ep.rule, v.w, mm.w, ms.w);
              *reinterpret_cast<float4*>(ep.upd_mom + off) = mm;
              *reinterpret_cast<float4*>(ep.upd_master + off) = ms;
              uint2 o;
              o.x = f2bf(ms.x) | ((uint32_t)f2bf(ms.y) << 16);
              o.y = f2bf(ms.z) | ((uint32_t)f2bf(ms.w) << 16);
              *reinterpret_cast<uint2*>(ep.upd_ring + off) = o;
            } else {
              *reinterpret_cast<float4*>(ep.out_f + off) = v;
            }
          }
        }
      } else {
        bf16_t* sb = reinterpret_cast<bf16_t*>(stage);  // [32][HLD]
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
          const int c = col_base + 32 * j + (l & 31);
          const float bv = (ep.bias && c < J) ? bf2f(ep.bias[c]) : 0.f;
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            float v = acc(i, j)[r] + bv;
            if (ep.relu) v = fmaxf(v, 0.f);
            sb[(8 * (r >> 2) + 4 * (l >> 5) + (r & 3)) * HLD + 32 * j + (l & 31)] = f2bf(v);
          }
        }
        constexpr int LPR = WCOLS / 8;       // lanes per row (8 bf16 each)
        constexpr int RPP = 64 / LPR;
#pragma unroll
        for (int q = 0; q < 32 / RPP; ++q) {
          const int rr = RPP * q + l / LPR, cc = (l % LPR) * 8;
          const int row = row_base + rr, c = col_base + cc;
          if (row < I && c < J) {
            uint4 v = *reinterpret_cast<const uint4*>(&sb[rr * HLD + cc]);
            const size_t off = (size_t)row * ep.ldo + c;
            if (ep.mask) {
              const uint4 mk = ldg16(ep.mask + off);
              const uint32_t mw[4] = {mk.x, mk.y, mk.z, mk.w};
              uint32_t vw[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                if (!bf_positive((uint16_t)(mw[e] & 0xffffu))) vw[e] &= 0xffff0000u;
                if (!bf_positive((uint16_t)(mw[e] >> 16))) vw[e] &= 0x0000ffffu;
              }
              v = make_uint4(vw[0], vw[1], vw[2], vw[3]);
            }
            *reinterpret_cast<uint4*>(ep.out + off) = v;
          }
        }
      }
    }
    return;
  }
  // odd widths: element-wise from the accumulators (column = lane, 16 rows per block)
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int c = col_base + 32 * j + (l & 31);
    if (c >= J) continue;
    const float bv = ep.bias ? bf2f(ep.bias[c]) : 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = row0 + 32 * i + 8 * (r >> 2) + 4 * (l >> 5) + (r & 3);
        if (row >= I) continue;
        float v = acc(i, j)[r] + bv;
        if (ep.relu) v = fmaxf(v, 0.f);
        const size_t off = (size_t)row * ep.ldo + c;
        if (ep.upd_master) {
          float m = ep.upd_mom[off], wv = ep.upd_master[off];
          apply_update(ep.rule, v, m, wv);
          ep.upd_mom[off] = m;
          ep.upd_master[off] = wv;
          ep.upd_ring[off] = f2bf(wv);
        } else if (ep.out_f) {
          ep.out_f[off] = v;
        } else {
          uint16_t o = f2bf(v);
          if (ep.mask && !bf_positive(ep.mask[off])) o = 0;
          ep.out[off] = o;
        }
      }
  }
}

// NW = waves per workgroup: 4 (2 x 2 waves of 128 x 128) or 8 (2 x 4 waves of 128 x 64, two waves per SIMD so
// that one can issue MFMAs while the other waits for LDS).
template <bool TA, bool TB, int NW>
__global__ __launch_bounds__(64 * NW, 1) void gemm_big_kernel(const bf16_t* __restrict__ A, int lda,
                                                              const bf16_t* __restrict__ Bm, int ldb, BigEpilogue ep,
                                                              int I, int J, int R) {
  constexpr int NT = 64 * NW;           // threads
  constexpr int WN = NW / 2;            // waves along the columns (2 along the rows)
  constexpr int NJ = (GN / WN) / 32;    // 32-column blocks per wave (4 or 2)
  constexpr int WCOLS = GN / WN;        // columns per wave
  constexpr int PCH = GM * 8 / NT;      // 16-byte chunks per thread, plain layout (8 or 4)
  constexpr int SCH = 1024 / NT;        // 2x8 blocks per thread, sideways layout (4 or 2)
  constexpr int kStageBytes = 147456 / NW;
  // one operand tile: 256 rows x 64 reduction elements; plain layout padded to GLD, transposed layout swizzled
  constexpr int kTile = GM * GLD;  // bf16 elements reserved per tile and buffer (the swizzled form needs 256*64)
  __shared__ __attribute__((aligned(16))) bf16_t smem[4 * kTile];
  bf16_t* const As0 = smem;
  bf16_t* const Bs0 = smem + 2 * kTile;
  const int t = threadIdx.x, l = t & 63, w = t >> 6, wm = w / WN, wn = w % WN;
  const int i0 = blockIdx.y * GM, j0 = blockIdx.x * GN;
  const int T = (R + GK - 1) / GK;

  struct Regs {
    uint4 a[PCH], b[PCH];
  };
  auto load_plain = [&](uint4* r, const bf16_t* src, int ld, int row0, int nrows, int st) {
    const int rr = st * GK + (t & 7) * 8;
#pragma unroll
    for (int i = 0; i < PCH; ++i) {
      const int row = row0 + (t >> 3) + (NT / 8) * i;
      r[i] = (st < T && row < nrows && rr < R) ? ldg16(src + (size_t)row * ld + rr) : zero16();
    }
  };
  auto load_sideways = [&](uint4* r, const bf16_t* src, int ld, int col0, int ncols, int st) {
#pragma unroll
    for (int i = 0; i < SCH; ++i) {
      // a wave: 8 column chunks x 8 reduction pairs
      const int cc = (((NT / 256) * i + (t >> 8)) << 3) | (t & 7), pair = (t >> 3) & 31;
      const int rr = st * GK + 2 * pair, c = col0 + 8 * cc;
      r[2 * i] = (st < T && rr < R && c < ncols) ? ldg16(src + (size_t)rr * ld + c) : zero16();
      r[2 * i + 1] = (st < T && rr + 1 < R && c < ncols) ? ldg16(src + (size_t)(rr + 1) * ld + c) : zero16();
    }
  };
  auto store_plain = [&](bf16_t* tile, const uint4* r) {
#pragma unroll
    for (int i = 0; i < PCH; ++i)
      *reinterpret_cast<uint4*>(&tile[((t >> 3) + (NT / 8) * i) * GLD + (t & 7) * 8]) = r[i];
  };
  auto store_sideways = [&](bf16_t* tile, const uint4* r) {
    uint32_t* tw = reinterpret_cast<uint32_t*>(tile);
#pragma unroll
    for (int i = 0; i < SCH; ++i) {
      const int cc = (((NT / 256) * i + (t >> 8)) << 3) | (t & 7), pair = (t >> 3) & 31;
      store_transposed_pair<8>(tw, 8 * cc, pair, r[2 * i], r[2 * i + 1]);
    }
  };
  auto gload = [&](Regs& r, int st) {
    if (TA) load_sideways(r.a, A, lda, i0, I, st); else load_plain(r.a, A, lda, i0, I, st);
    if (TB) load_sideways(r.b, Bm, ldb, j0, J, st); else load_plain(r.b, Bm, ldb, j0, J, st);
  };
  auto sstore = [&](int buf, const Regs& r) {
    if (TA) store_sideways(As0 + buf * kTile, r.a); else store_plain(As0 + buf * kTile, r.a);
    if (TB) store_sideways(Bs0 + buf * kTile, r.b); else store_plain(Bs0 + buf * kTile, r.b);
  };

  f32x16 acc[4][NJ];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j) acc[i][j] = f32x16{0};

  Regs Rg;
  gload(Rg, 0);
  sstore(0, Rg);
  __syncthreads();
  for (int st = 0; st < T; ++st) {
    const int cur = st & 1;
    gload(Rg, st + 1);
    const bf16_t* as = As0 + cur * kTile;
    const bf16_t* bs = Bs0 + cur * kTile;
#pragma unroll
    for (int ks = 0; ks < GK / 16; ++ks) {
      const int kk = ks * 16 + (l >> 5) * 8, grp = 2 * ks + (l >> 5);
      uint4 a[4], b[NJ];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = 128 * wm + 32 * i + (l & 31);
        a[i] = TA ? load_swizzled_frag<8>(reinterpret_cast<const uint32_t*>(as), row, grp)
                  : *reinterpret_cast<const uint4*>(&as[row * GLD + kk]);
      }
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        const int row = WCOLS * wn + 32 * j + (l & 31);
        b[j] = TB ? load_swizzled_frag<8>(reinterpret_cast<const uint32_t*>(bs), row, grp)
                  : *reinterpret_cast<const uint4*>(&bs[row * GLD + kk]);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(a[i]), frag(b[j]), acc[i][j], 0, 0, 0);
    }
    if (st + 1 < T) sstore(cur ^ 1, Rg);
    __syncthreads();
  }

  char* const est = reinterpret_cast<char*>(smem) + (size_t)w * kStageBytes;
  if constexpr (NJ == 2) {
    big_epilogue<2, 64>(acc, ep, est, i0 + 128 * wm, j0 + WCOLS * wn, l, I, J);
  } else {
    big_epilogue<2, 64, NJ, 0>(acc, ep, est, i0 + 128 * wm, j0 + WCOLS * wn, l, I, J);
    big_epilogue<2, 64, NJ, 2>(acc, ep, est, i0 + 128 * wm, j0 + WCOLS * wn + 64, l, I, J);
  }
}

// ---- both operands reduction-contiguous: global -> LDS without passing through registers --------------------
// Same 256 x 256 tile and 2 x 4 waves of 128 x 64, but 32 reduction elements per stage and four stages in LDS.
// Each lane's 16-byte chunk goes straight from global memory into LDS (global_load_lds_dwordx4); the hardware
// places lane L's chunk at M0 + 16 L, so a wave-wide load fills 16 consecutive 64-byte tile rows and the XOR
// swizzle of a row's four 16-byte slots is applied on the global side (lane L fetches the k-group that belongs in
// its slot).  The loads of stage st+3 are spread between the MFMAs of stage st; the barrier at the end of stage
// st publishes stage st+2, and the first fragments of stage st+1 are already in registers when it is reached.
// The loads are written as inline assembly: for the builtin the compiler inserts a wait for ALL outstanding loads
// before every LDS read, which serialises the pipeline.  A reduction length that is not a multiple of 32 is
// handled by one zero-padded stage that goes through registers before the pipeline starts.
constexpr int DK = 32, DNS = 4, DROWB = DK * 2, DTILE = 256 * DROWB, DSTAGE = 2 * DTILE;
__device__ __forceinline__ int dma_swz(int row) { return (row >> 2) & 3; }

// NW = 8: 2 x 4 waves of 128 x 64 (two waves per SIMD: one issues MFMAs while the other waits; 0.75 LDS fragment
// reads per MFMA).  NW = 4: 2 x 2 waves of 128 x 128 (one wave per SIMD, 0.5 fragment reads per MFMA, which is what
// the LDS read path can sustain at the full MFMA rate); with a single wave per SIMD nothing hides a stall, so the
// order of MFMAs, fragment reads and loads inside a reduction step is pinned: one memory instruction behind each of
// the first twelve MFMAs of the step's sixteen.
template <int NW>
__global__ __launch_bounds__(64 * NW, 1) void gemm_dma_kernel(const bf16_t* __restrict__ A, int lda,
                                                              const bf16_t* __restrict__ Bm, int ldb, BigEpilogue ep,
                                                              int I, int J, int R, int tiles_i, int tiles_j) {
  constexpr int NT = 64 * NW, WN = NW / 2, WCOLS = 256 / WN;
  constexpr int NI = 4, NJ = WCOLS / 32, KS = DK / 16, D = DNS - 1;
  constexpr int QN = 256 / 16 / NW;        // wave-wide loads per operand and stage (2 or 4)
  constexpr int LPS = 2 * QN, LPK = LPS / KS, MF = NI * NJ;
  __shared__ __attribute__((aligned(1024))) char smem[DNS * DSTAGE];
  const int t = threadIdx.x, l = t & 63;
  const int w = __builtin_amdgcn_readfirstlane(t >> 6), wm = w / WN, wn = w % WN;
  // Workgroups are dealt round-robin to the 8 XCDs (each with its own L2): renumber so that an XCD works on a
  // contiguous run of tiles, and walk the tiles in bands of four tile rows so that the tiles in flight on one XCD
  // share a few A and B panels.
  int bid = blockIdx.x;
  {
    const int per = gridDim.x >> 3;
    if (bid < per * 8) bid = (bid & 7) * per + (bid >> 3);
  }
  int ti, tj;
  {
    constexpr int BAND = 4;
    const int per_band = BAND * tiles_j, band = bid / per_band, rem = bid - band * per_band;
    const int rows_in = tiles_i - band * BAND < BAND ? tiles_i - band * BAND : BAND;
    ti = band * BAND + rem % rows_in;
    tj = rem / rows_in;
  }
  const int i0 = ti * GM, j0 = tj * GN;
  const int T = R / DK, tail = R - T * DK;  // T >= 1 (checked by the launcher)

  // byte offsets of this lane's chunk for each of the stage's loads (A loads first); rows beyond the matrix are
  // clamped to its last row: they only feed outputs that are never stored
  uint32_t off[LPS];
#pragma unroll
  for (int q = 0; q < QN; ++q) {
    const int row = (q * NW + w) * 16 + (l >> 2), g = (l & 3) ^ dma_swz(row);
    const int ra = i0 + row < I ? i0 + row : I - 1, rb = j0 + row < J ? j0 + row : J - 1;
    off[q] = ((uint32_t)ra * (uint32_t)lda + g * 8) * 2u;
    off[QN + q] = ((uint32_t)rb * (uint32_t)ldb + g * 8) * 2u;
  }
  auto load1 = [&](int q, char* stage, int k0) {  // q-th load of the stage that starts at reduction index k0
    dma_load16((q < QN ? A : Bm) + k0, off[q], stage + (q < QN ? 0 : DTILE) + ((q % QN) * NW + w) * 1024);
  };

  f32x16 acc[NI][NJ];
#pragma unroll
  for (int i = 0; i < NI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j) acc[i][j] = f32x16{0};
  // byte offsets of this lane's fragments inside a stage for k-step 0; k-step 1 flips bit 5 (two slots further)
  int fa[NI], fb[NJ];
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const int row = 128 * wm + 32 * i + (l & 31);
    fa[i] = row * DROWB + (((l >> 5) ^ dma_swz(row)) << 4);
  }
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int row = WCOLS * wn + 32 * j + (l & 31);
    fb[j] = DTILE + row * DROWB + (((l >> 5) ^ dma_swz(row)) << 4);
  }
  auto ldf = [&](const char* stage, int o, int ks) { return *reinterpret_cast<const uint4*>(stage + (o ^ (ks << 5))); };

#pragma unroll
  for (int d = 0; d < D; ++d) {
    const int sc = d < T ? d : T - 1;
#pragma unroll
    for (int q = 0; q < LPS; ++q) load1(q, smem + d * DSTAGE, sc * DK);
  }
  if (tail) {  // ragged end of the reduction: through registers with zero fill, into the stage the pipeline fills last
    char* st = smem + D * DSTAGE;
#pragma unroll
    for (int i = 0; i < 1024 / NT; ++i) {
      const int c = t + NT * i, row = c >> 2, g = c & 3, k = T * DK + g * 8;
      const int ra = i0 + row < I ? i0 + row : I - 1, rb = j0 + row < J ? j0 + row : J - 1;
      const uint4 va = k < R ? ldg16(A + (size_t)ra * lda + k) : zero16();
      const uint4 vb = k < R ? ldg16(Bm + (size_t)rb * ldb + k) : zero16();
      const int o = row * DROWB + ((g ^ dma_swz(row)) << 4);
      *reinterpret_cast<uint4*>(st + o) = va;
      *reinterpret_cast<uint4*>(st + DTILE + o) = vb;
    }
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      uint4 a[NI], b[NJ];
#pragma unroll
      for (int i = 0; i < NI; ++i) a[i] = ldf(st, fa[i], ks);
#pragma unroll
      for (int j = 0; j < NJ; ++j) b[j] = ldf(st, fb[j], ks);
#pragma unroll
      for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(a[i]), frag(b[j]), acc[i][j], 0, 0, 0);
    }
  }
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"((D - 2) * LPS) : "memory");  // stages 0 and 1 have landed
  __syncthreads();  // (also: every wave is done with the ragged stage before the loop's first loads overwrite it)
  uint4 a[2][NI], b[2][NJ];
#pragma unroll
  for (int i = 0; i < NI; ++i) a[0][i] = ldf(smem, fa[i], 0);
#pragma unroll
  for (int j = 0; j < NJ; ++j) b[0][j] = ldf(smem, fb[j], 0);
  int cur = 0, fill = D;  // LDS stage of reduction stage st; LDS stage this iteration's loads go to
  for (int st = 0; st < T; ++st) {
    const char* sc = smem + cur * DSTAGE;
    cur = cur + 1 == DNS ? 0 : cur + 1;
    const char* sn = smem + cur * DSTAGE;
    char* sl = smem + fill * DSTAGE;
    fill = fill + 1 == DNS ? 0 : fill + 1;
    const int k0 = (st + D < T ? st + D : T - 1) * DK;  // past the end: reload the last stage (never read)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int c = ks & 1, n = c ^ 1;
      const char* src = ks + 1 < KS ? sc : sn;  // next step's fragments; the next stage was published a barrier ago
      const int kn = ks + 1 < KS ? ks + 1 : 0;
      if constexpr (NW == 8) {
#pragma unroll
        for (int i = 0; i < NI; ++i) a[n][i] = ldf(src, fa[i], kn);
#pragma unroll
        for (int j = 0; j < NJ; ++j) b[n][j] = ldf(src, fb[j], kn);
#pragma unroll
        for (int m = 0; m < MF; ++m) {
          const int i = m / NJ, j = m % NJ;
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(a[c][i]), frag(b[c][j]), acc[i][j], 0, 0, 0);
#pragma unroll
          for (int x = 0; x < LPK; ++x)
            if (m == x * MF / LPK + 1) {
              __builtin_amdgcn_sched_barrier(0);
              load1(ks * LPK + x, sl, k0);
              __builtin_amdgcn_sched_barrier(0);
            }
        }
      } else {
        // sixteen MFMAs; behind MFMA m: m % 3 != 2 -> the next fragment read (eight in all), m % 3 == 2 -> the next
        // global -> LDS load (four), m >= 12 -> nothing
#pragma unroll
        for (int m = 0; m < MF; ++m) {
          const int i = m / NJ, j = m % NJ;
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(a[c][i]), frag(b[c][j]), acc[i][j], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
          if (m < 12) {
            if (m % 3 == 2) {
              load1(ks * LPK + m / 3, sl, k0);
            } else {
              // in the order the next step's MFMAs need them: A0, B0..B3 (MFMAs 0-3), then A1, A2, A3
              const int f = m - m / 3;  // 0..7
              if (f == 0) a[n][0] = ldf(src, fa[0], kn);
              else if (f <= NJ) b[n][f - 1] = ldf(src, fb[f - 1], kn);
              else a[n][f - NJ] = ldf(src, fa[f - NJ], kn);
            }
            __builtin_amdgcn_sched_barrier(0);
          }
        }
      }
    }
    // this wave's loads of stage st+2 have landed (those of stage st+3 may still be in flight); after the barrier
    // every wave's have, and every wave is done reading stage st
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"((D - 2) * LPS) : "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  char* const est = smem + (size_t)w * (DNS * DSTAGE / NW);
  if constexpr (NJ == 2) {
    big_epilogue<2, 64>(acc, ep, est, i0 + 128 * wm, j0 + WCOLS * wn, l, I, J);
  } else {
    big_epilogue<2, 64, NJ, 0>(acc, ep, est, i0 + 128 * wm, j0 + WCOLS * wn, l, I, J);
    big_epilogue<2, 64, NJ, 2>(acc, ep, est, i0 + 128 * wm, j0 + WCOLS * wn + 64, l, I, J);
  }
}

// ---- the same product with 128-byte tile rows -----------------------------------------------------------------
// 64 reduction elements per stage: a tile row is one whole 128-byte cache line, so a wave-wide global -> LDS load
// touches 8 lines instead of 16 (the L2 -> compute-unit path moves whole lines half as often per byte).  An operand
// tile of a stage is 256 rows x 128 bytes = 32 KB; LDS holds a ring of five such tiles (160 KB), filled in the order
// A(0) B(0) A(1) B(1) A(2) ...  A stage's compute reads two of them; the other three are in flight or landed.
// The stage barrier sits in front of a stage's LAST reduction step: by then the wave holds that step's fragments in
// registers, so the barrier both publishes stage st+1 (this wave's loads of B(st+1) have landed, A(st+1) landed a
// stage earlier) and frees the two tiles of stage st, into which B(st+2) and A(st+3) are loaded during the last step
// of stage st and the first three of stage st+1; the first fragments of stage st+1 are read behind the barrier, under
// the MFMAs of the last step.  Needs R % 64 == 0 and R >= 128.
// What bounds it (four waves, 8192 x 4096 x 25088, 56 % of the nominal peak): with the global -> LDS loads taken out
// of the main loop the MFMAs and fragment reads alone run at 74-80 %; with the loads in, 56 %, also when every load
// hits the same cached 64 KB, no faster with half of the fragment reads removed, and SLOWER (52 %) with B fetched
// through registers and written with ds_write_b128 so that only A uses the direct path.  The hardware counters add the
// other half of the picture: the matrix pipes are busy in 77 % of the cycles, but the chip runs these launches at
// 1.7 GHz instead of its nominal 2.4 (on all-zero operands, which draw less power, the same kernel reaches 73 % of the
// nominal peak), so what is gained in issue efficiency is partly paid back in clock.
constexpr int EK = 64, EROWB = 128, ETILE = 256 * EROWB, ERING = 5;
// Slot swizzle of a 128-byte row.  A 16-byte-per-lane LDS read is served 16 consecutive lanes (256 bytes, all 64
// banks) at a time; those lanes read the same logical slot of 16 consecutive rows.  Two rows fill the 64 banks, so
// the physical slot has to differ between the eight rows of equal parity: slot ^ ((row >> 1) & 7).  (slot ^ (row & 7)
// puts rows r and r + 8 on the same banks: measured as one bank-conflict cycle per LDS cycle.)
__device__ __forceinline__ int e_swz(int row) { return (row >> 1) & 7; }

template <int NW>
__global__ __launch_bounds__(64 * NW, 1) void gemm_dma64_kernel(const bf16_t* __restrict__ A, int lda,
                                                                const bf16_t* __restrict__ Bm, int ldb, BigEpilogue ep,
                                                                int I, int J, int R, int tiles_i, int tiles_j,
                                                                int splits, float* __restrict__ part) {
  constexpr int WN = NW / 2, WCOLS = 256 / WN;
  constexpr int NI = 4, NJ = WCOLS / 32, KS = EK / 16, MF = NI * NJ;
  constexpr int QN = 32 / NW;              // wave-wide loads per wave and operand tile (4 or 8): 8 rows each
  constexpr int LPK = 2 * QN / KS;         // loads behind the MFMAs of one reduction step (2 or 4)
  __shared__ __attribute__((aligned(1024))) char smem[ERING * ETILE];
  const int t = threadIdx.x, l = t & 63;
  const int w = __builtin_amdgcn_readfirstlane(t >> 6), wm = w / WN, wn = w % WN;
  // splits > 1: the grid holds `splits` copies of the tile grid; copy z reduces its share of the stages and leaves an
  // fp32 partial product in part[z][I][J] (no bias, activation or rounding: the reducing kernel applies them)
  const int n_tiles = tiles_i * tiles_j;
  const int z = blockIdx.x / n_tiles;
  int bid = blockIdx.x - z * n_tiles;
  {
    const int per = n_tiles >> 3;
    if (bid < per * 8) bid = (bid & 7) * per + (bid >> 3);
  }
  int ti, tj;
  {
    constexpr int BAND = 4;
    const int per_band = BAND * tiles_j, band = bid / per_band, rem = bid - band * per_band;
    const int rows_in = tiles_i - band * BAND < BAND ? tiles_i - band * BAND : BAND;
    ti = band * BAND + rem % rows_in;
    tj = rem / rows_in;
  }
  const int i0 = ti * GM, j0 = tj * GN;
  int T = R / EK;
  if (splits > 1) {
    const int s0 = (int)((long long)z * T / splits), s1 = (int)((long long)(z + 1) * T / splits);
    A += (size_t)s0 * EK;
    Bm += (size_t)s0 * EK;
    T = s1 - s0;
    ep.bias = nullptr; ep.mask = nullptr; ep.relu = 0; ep.out = nullptr; ep.upd_master = nullptr;
    ep.out_f = part + (size_t)z * I * J;
    ep.ldo = J;
  }

  // this lane's chunk in each of a tile's loads: 8 lanes per row, the XOR swizzle of the row's eight 16-byte slots
  // applied on the global side; rows beyond the matrix are clamped (they only feed outputs that are never stored)
  uint32_t offa[QN], offb[QN];
#pragma unroll
  for (int q = 0; q < QN; ++q) {
    const int row = (q * NW + w) * 8 + (l >> 3), g = (l & 7) ^ e_swz(row);
    const int ra = i0 + row < I ? i0 + row : I - 1, rb = j0 + row < J ? j0 + row : J - 1;
    offa[q] = ((uint32_t)ra * (uint32_t)lda + g * 8) * 2u;
    offb[q] = ((uint32_t)rb * (uint32_t)ldb + g * 8) * 2u;
  }
  const uint32_t lds0 = lds_address_of(smem) + (uint32_t)w * 1024u;  // this wave's first destination in ring slot 0
  auto load_a = [&](int q, int slot, int stage) {
    dma_load16_at(A + (stage < T ? stage : T - 1) * EK, offa[q], lds0 + (uint32_t)(slot * ETILE + q * NW * 1024));
  };
  auto load_b = [&](int q, int slot, int stage) {
    dma_load16_at(Bm + (stage < T ? stage : T - 1) * EK, offb[q], lds0 + (uint32_t)(slot * ETILE + q * NW * 1024));
  };

  f32x16 acc[NI][NJ];
#pragma unroll
  for (int i = 0; i < NI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j) acc[i][j] = f32x16{0};
  // byte offsets of this lane's fragments inside a tile for reduction step 0; step ks flips bits 5 and 6 by ks
  int fa[NI], fb[NJ];
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const int row = 128 * wm + 32 * i + (l & 31);
    fa[i] = row * EROWB + (((l >> 5) ^ e_swz(row)) << 4);
  }
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int row = WCOLS * wn + 32 * j + (l & 31);
    fb[j] = row * EROWB + (((l >> 5) ^ e_swz(row)) << 4);
  }
  auto ldf = [&](const char* tile, int o, int ks) { return *reinterpret_cast<const uint4*>(tile + (o ^ (ks << 5))); };

  // prologue: A(0) B(0) A(1) and the first half of B(1) (what the last step of a stage "-1" would have issued)
#pragma unroll
  for (int q = 0; q < QN; ++q) load_a(q, 0, 0);
#pragma unroll
  for (int q = 0; q < QN; ++q) load_b(q, 1, 0);
#pragma unroll
  for (int q = 0; q < QN; ++q) load_a(q, 2, 1);
#pragma unroll
  for (int q = 0; q < LPK; ++q) load_b(q, 3, 1);
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(QN + LPK) : "memory");  // A(0) and B(0) have landed
  __syncthreads();
  uint4 a[2][NI], b[2][NJ];
#pragma unroll
  for (int i = 0; i < NI; ++i) a[0][i] = ldf(smem, fa[i], 0);
#pragma unroll
  for (int j = 0; j < NJ; ++j) b[0][j] = ldf(smem + ETILE, fb[j], 0);
  int sa = 0;  // ring slot of A(st); B(st) is the next one, A(st+1) the one after, ...
  auto ring = [](int x) { return x >= ERING ? x - ERING : x; };
  for (int st = 0; st < T; ++st) {
    const int sb = ring(sa + 1), sa1 = ring(sa + 2), sb1 = ring(sa + 3), sa2 = ring(sa + 4);
    const char* ta = smem + sa * ETILE;
    const char* tb = smem + sb * ETILE;
    const char* ta1 = smem + sa1 * ETILE;
    const char* tb1 = smem + sb1 * ETILE;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int c = ks & 1, n = c ^ 1;
      if (ks == KS - 1) {
        // this wave holds its last fragments of stage st; its loads of B(st+1) have landed (A(st+2)'s may be in flight)
        asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(QN) : "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
      }
      const char* pa = ks + 1 < KS ? ta : ta1;  // where the next step's fragments lie
      const char* pb = ks + 1 < KS ? tb : tb1;
      const int kn = ks + 1 < KS ? ks + 1 : 0;
      if constexpr (NW == 8) {
#pragma unroll
        for (int i = 0; i < NI; ++i) a[n][i] = ldf(pa, fa[i], kn);
#pragma unroll
        for (int j = 0; j < NJ; ++j) b[n][j] = ldf(pb, fb[j], kn);
      }
#pragma unroll
      for (int m = 0; m < MF; ++m) {
        const int i = m / NJ, j = m % NJ;
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(a[c][i]), frag(b[c][j]), acc[i][j], 0, 0, 0);
        int x = -1;  // which of the step's loads goes behind this MFMA (-1: none)
        if constexpr (NW == 8) {
          if (m == 1) x = 0;
          if (m == 5) x = 1;
        } else {
          __builtin_amdgcn_sched_barrier(0);
          if (m < 12) {
            if (m % 3 == 2) {
              x = m / 3;
            } else {
              const int f = m - m / 3;  // 0..7, in the order the next step's MFMAs need them: A0, B0..B3, A1..A3
              if (f == 0) a[n][0] = ldf(pa, fa[0], kn);
              else if (f <= NJ) b[n][f - 1] = ldf(pb, fb[f - 1], kn);
              else a[n][f - NJ] = ldf(pa, fa[f - NJ], kn);
              __builtin_amdgcn_sched_barrier(0);
            }
          }
        }
        if (x >= 0) {
          __builtin_amdgcn_sched_barrier(0);
          // Loads between two barriers, in issue order: B(s+1) first half (last step of stage s-1), B(s+1) second
          // half (step 0 of stage s), A(s+2) first half (step 1), A(s+2) second half (step 2).  With sa the slot of
          // A(st): B(st+1) lives in ring(sa + 3), A(st+2) in ring(sa + 4), B(st+2) in ring(sa + 5) = sa.
          if (ks == KS - 1) load_b(x, sa, st + 2);
          else if (ks == 0) load_b(LPK + x, sb1, st + 1);
          else if (ks == 1) load_a(x, sa2, st + 2);
          else load_a(LPK + x, sa2, st + 2);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
    sa = sa1;
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  char* const est = smem + (size_t)w * (ERING * ETILE / NW);
  if constexpr (NJ == 2) {
    big_epilogue<2, 64>(acc, ep, est, i0 + 128 * wm, j0 + WCOLS * wn, l, I, J);
  } else {
    big_epilogue<2, 64, NJ, 0>(acc, ep, est, i0 + 128 * wm, j0 + WCOLS * wn, l, I, J);
    big_epilogue<2, 64, NJ, 2>(acc, ep, est, i0 + 128 * wm, j0 + WCOLS * wn + 64, l, I, J);
  }
}

// ---- both operands stored with the reduction index as their slow axis (the weight gradient) --------------------
//   out[n][k] = sum over rows m of z[m][n] * x[m][k]          z: [M][N], x: [M][K], out: [N][K] fp32
// The tiles go into LDS as they lie in memory ([32 rows][256 columns] per operand and stage, straight from global
// memory, 16 bytes per lane) and the MFMA operands are fetched with the transposing LDS read ds_read_b64_tr_b16:
// in a group of 16 lanes, source lane j supplies the address of 4 columns (j % 4) of row (j / 4), lane i receives
// column i of those 4 rows -- "column i, 4 reduction elements" of a 32x32x16 operand.  No transposing pre-pass, no
// transposing stores.  256 x 256 output tile, 8 waves of 128 x 64, four stages, loads three stages ahead; rows past
// M and columns past N / K are fetched from a block of zeros.  A row of a tile is 512 bytes = 8 slots of 64 bytes
// (32 columns); slot s of row r holds column block s ^ (r & 3), so that the 4 rows one transposing read touches
// fall into different banks.
__device__ __attribute__((aligned(16))) const uint32_t g_tn_zero[4] = {0u, 0u, 0u, 0u};
typedef short tn_v4i16_t __attribute__((ext_vector_type(4)));
typedef short tn_v8i16_t __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) tn_v4i16_t tn_lds_v4i16_t;

#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void dma_chunk64(const bf16_t* lane_src, char* uniform_lds_dst) {
  const uint32_t lds_addr = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_void_t*)(uniform_lds_dst));
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(lane_src), "s"(lds_addr) : "memory", "m0");
}
__device__ __forceinline__ void dma_chunk64_at(const bf16_t* lane_src, uint32_t uniform_lds_addr) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(lane_src), "s"(uniform_lds_addr) : "memory", "m0");
}
#pragma clang diagnostic pop
__device__ __forceinline__ bf16x8 tn_frag(const char* lo, const char* hi) {
  const tn_v4i16_t a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((tn_lds_v4i16_t*)lo);
  const tn_v4i16_t b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((tn_lds_v4i16_t*)hi);
  const tn_v8i16_t v = __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, v);
}

// logical tile number -> tile coordinates: bands of four tile rows, walked column by column (neighbouring numbers
// share operand panels in L2)
__device__ __forceinline__ void tn_tile_of(int bid, int tiles_n, int tiles_k, int& tn, int& tk) {
  constexpr int BAND = 4;
  const int per_band = BAND * tiles_k, band = bid / per_band, rem = bid - band * per_band;
  const int rows_in = tiles_n - band * BAND < BAND ? tiles_n - band * BAND : BAND;
  tn = band * BAND + rem % rows_in;
  tk = rem / rows_in;
}

// The tiles whose rows gemm_tn_kernel split (tail_splits partial tiles each): add the partial tiles in split order
// and apply the update.  64 workgroups per tile, four elements per lane.
__global__ __launch_bounds__(256) void tn_tail_update_kernel(const float* __restrict__ part, int n_tail, int splits,
                                                             int tail_first, int tiles_n, int tiles_k, int N, int K,
                                                             float* __restrict__ master, float* __restrict__ mom,
                                                             bf16_t* __restrict__ ring, UpdateRule rule) {
  const int t_i = blockIdx.x >> 6;
  const int idx = ((blockIdx.x & 63) * 256 + threadIdx.x) * 4;  // element of the 256 x 256 tile
  int tn, tk;
  tn_tile_of(tail_first + t_i, tiles_n, tiles_k, tn, tk);
  const int row = tn * GM + idx / GN, col = tk * GN + idx % GN;
  if (row >= N || col >= K) return;  // (K is a multiple of 8: four columns are inside or outside together)
  float4 g = *reinterpret_cast<const float4*>(part + (size_t)t_i * (GM * GN) + idx);
  for (int z = 1; z < splits; ++z) {
    const float4 p = *reinterpret_cast<const float4*>(part + ((size_t)z * n_tail + t_i) * (GM * GN) + idx);
    g.x += p.x; g.y += p.y; g.z += p.z; g.w += p.w;
  }
  const size_t off = (size_t)row * K + col;
  float4 mm = *reinterpret_cast<const float4*>(mom + off);
  float4 ms = *reinterpret_cast<const float4*>(master + off);
  apply_update(rule, g.x, mm.x, ms.x); apply_update(rule, g.y, mm.y, ms.y);
  apply_update(rule, g.z, mm.z, ms.z); apply_update(rule, g.w, mm.w, ms.w);
  *reinterpret_cast<float4*>(mom + off) = mm;
  *reinterpret_cast<float4*>(master + off) = ms;
  uint2 o;
  o.x = f2bf_pair(ms.x, ms.y);
  o.y = f2bf_pair(ms.z, ms.w);
  *reinterpret_cast<uint2*>(ring + off) = o;
}

// The same for an input gradient (gemm_nt_kernel's tail tiles): partial tiles added in split order, the ReLU mask of
// the producing layer applied, rounded to bf16.
__global__ __launch_bounds__(256) void nt_tail_store_kernel(const float* __restrict__ part, int n_tail, int splits,
                                                            int tail_first, int tiles_i, int tiles_j, int I, int J,
                                                            const bf16_t* __restrict__ mask, bf16_t* __restrict__ out) {
  const int t_i = blockIdx.x >> 6;
  const int idx = ((blockIdx.x & 63) * 256 + threadIdx.x) * 4;
  int ti, tj;
  tn_tile_of(tail_first + t_i, tiles_i, tiles_j, ti, tj);
  const int row = ti * GM + idx / GN, col = tj * GN + idx % GN;
  if (row >= I || col >= J) return;  // (J is a multiple of 8)
  float4 g = *reinterpret_cast<const float4*>(part + (size_t)t_i * (GM * GN) + idx);
  for (int z = 1; z < splits; ++z) {
    const float4 p = *reinterpret_cast<const float4*>(part + ((size_t)z * n_tail + t_i) * (GM * GN) + idx);
    g.x += p.x; g.y += p.y; g.z += p.z; g.w += p.w;
  }
  const size_t off = (size_t)row * J + col;
  uint2 o;
  o.x = f2bf_pair(g.x, g.y);
  o.y = f2bf_pair(g.z, g.w);
  if (mask) {
    const uint2 mk = *reinterpret_cast<const uint2*>(mask + off);
    if (!bf_positive((uint16_t)(mk.x & 0xffffu))) o.x &= 0xffff0000u;
    if (!bf_positive((uint16_t)(mk.x >> 16))) o.x &= 0x0000ffffu;
    if (!bf_positive((uint16_t)(mk.y & 0xffffu))) o.y &= 0xffff0000u;
    if (!bf_positive((uint16_t)(mk.y >> 16))) o.y &= 0x0000ffffu;
  }
  *reinterpret_cast<uint2*>(out + off) = o;
}

__global__ __launch_bounds__(512, 1) void gemm_tn_kernel(const bf16_t* __restrict__ Z, int ldz,
                                                         const bf16_t* __restrict__ X, int ldx, BigEpilogue ep, int M,
                                                         int N, int K, int tiles_n, int tiles_k, int splits,
                                                         float* __restrict__ part, int tail_first, int tail_splits) {
  constexpr int NW = 8, NI = 4, NJ = 2, TR = 32, KS = TR / 16, NS = 4, D = NS - 1;
  constexpr int ROWB = 512, TILE = TR * ROWB, STAGE = 2 * TILE;  // 16 KB per operand and stage
  constexpr int LPS = 2 * TILE / 1024 / NW;                      // wave-wide loads per wave and stage (4)
  constexpr int MF = NI * NJ;
  __shared__ __attribute__((aligned(1024))) char smem[NS * STAGE];
  const int t = threadIdx.x, l = t & 63;
  const int w = __builtin_amdgcn_readfirstlane(t >> 6), wm = w >> 2, wn = w & 3;
  // splits > 1: the grid holds `splits` copies of the tile grid; copy z sums over its share of the rows and leaves an
  // fp32 partial gradient in part[z][N][K] (no update: the reducing kernel applies it)
  // tail_splits > 1 (with splits == 1): tiles [0, tail_first) -- a whole number of rounds of the chip -- are computed
  // as usual with the update in the store; each of the remaining tiles is computed by tail_splits workgroups over
  // shares of the rows, which leave fp32 partial tiles in part[z][tail tile][256][256] for tn_tail_update_kernel.
  // The last round of a launch whose tile count is a little over a multiple of the compute units would otherwise run
  // on a fraction of the chip for a whole tile's time.
  const int n_tiles = tiles_n * tiles_k;
  int z, bid, my_splits = splits, tail_tile = -1;
  if (tail_splits > 1 && (int)blockIdx.x >= tail_first) {
    const int e = (int)blockIdx.x - tail_first, r = n_tiles - tail_first;
    tail_tile = e % r;
    z = e / r;
    bid = tail_first + tail_tile;
    my_splits = tail_splits;
  } else {
    const int span = tail_splits > 1 ? tail_first : n_tiles;
    z = blockIdx.x / span;
    bid = blockIdx.x - z * span;
    const int per = span >> 3;
    if (bid < per * 8) bid = (bid & 7) * per + (bid >> 3);
  }
  int tn, tk;
  tn_tile_of(bid, tiles_n, tiles_k, tn, tk);
  const int n0 = tn * GM, k0 = tk * GN;
  int T = (M + TR - 1) / TR;
  int m_lo = 0, m_hi = M;  // this copy's rows
  if (my_splits > 1) {
    const int s0 = (int)((long long)z * T / my_splits), s1 = (int)((long long)(z + 1) * T / my_splits);
    m_lo = s0 * TR;
    m_hi = s1 * TR < M ? s1 * TR : M;
    T = s1 - s0;
    ep.bias = nullptr; ep.mask = nullptr; ep.relu = 0; ep.out = nullptr; ep.upd_master = nullptr;
    if (tail_tile >= 0) {  // a dense 256 x 256 tile of its own (the epilogue adds the tile's origin to its offsets)
      ep.out_f = part + ((size_t)z * (n_tiles - tail_first) + tail_tile) * (GM * GN) - ((ptrdiff_t)n0 * GN + k0);
      ep.ldo = GN;
    } else {
      ep.out_f = part + (size_t)z * N * K;
      ep.ldo = K;
    }
  }
  const bf16_t* const zero = reinterpret_cast<const bf16_t*>(g_tn_zero);

  // loads: per stage 16 wave-loads per operand, each two tile rows of 512 bytes; wave w issues numbers w, w + 8, ...
  const bf16_t* lp[LPS];  // this lane's source for stage 0 (null: column outside the matrix)
  int lrow[LPS], ldst[LPS];
  size_t lstep[LPS];
#pragma unroll
  for (int q = 0; q < LPS; ++q) {
    const int id = q * NW + w;                 // 0..15: z, 16..31: x
    const bool is_x = id >= 16;
    const int r = 2 * (id & 15) + (l >> 5);    // tile row (reduction index inside the stage)
    const int s16 = l & 31, blk = (s16 >> 2) ^ (r & 3);
    const int col = (is_x ? k0 : n0) + 32 * blk + 8 * (s16 & 3);
    const int ld = is_x ? ldx : ldz;
    lp[q] = col < (is_x ? K : N) ? (is_x ? X : Z) + (size_t)(m_lo + r) * ld + col : nullptr;
    lrow[q] = m_lo + r;
    lstep[q] = (size_t)TR * ld;
    ldst[q] = (is_x ? TILE : 0) + (id & 15) * 1024;
  }
  const uint32_t lds_base = lds_address_of(smem);
  auto issue = [&](int q, char* stage) {  // q-th load of this wave for the next stage to be fetched; advances
    const bool ok = lp[q] != nullptr && lrow[q] < m_hi;
    dma_chunk64_at(ok ? lp[q] : zero, lds_base + (uint32_t)(stage - smem) + (uint32_t)ldst[q]);
    if (lp[q] != nullptr) lp[q] += lstep[q];
    lrow[q] += TR;
  };

  const int mrow = 8 * (l >> 5) + ((l >> 2) & 3);
  const int chb = (16 * ((l >> 4) & 1) + 4 * (l & 3)) * 2;
  int fa[NI], fb[NJ];
#pragma unroll
  for (int i = 0; i < NI; ++i) fa[i] = mrow * ROWB + 64 * ((4 * wm + i) ^ (mrow & 3)) + chb;
#pragma unroll
  for (int j = 0; j < NJ; ++j) fb[j] = TILE + mrow * ROWB + 64 * ((2 * wn + j) ^ (mrow & 3)) + chb;
  auto lda_ = [&](const char* stage, int o, int ks) { return tn_frag(stage + o + 16 * ks * ROWB, stage + o + (16 * ks + 4) * ROWB); };

  f32x16 acc[NI][NJ];
#pragma unroll
  for (int i = 0; i < NI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j) acc[i][j] = f32x16{0};

#pragma unroll
  for (int d = 0; d < D; ++d)
#pragma unroll
    for (int q = 0; q < LPS; ++q) issue(q, smem + d * STAGE);
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"((D - 2) * LPS) : "memory");  // stages 0 and 1 have landed
  __syncthreads();
  bf16x8 a[2][NI], b[2][NJ];
#pragma unroll
  for (int i = 0; i < NI; ++i) a[0][i] = lda_(smem, fa[i], 0);
#pragma unroll
  for (int j = 0; j < NJ; ++j) b[0][j] = lda_(smem, fb[j], 0);
  int cur = 0, fill = D;
  for (int st = 0; st < T; ++st) {
    const char* sc = smem + cur * STAGE;
    cur = cur + 1 == NS ? 0 : cur + 1;
    const char* sn = smem + cur * STAGE;
    char* sl = smem + fill * STAGE;
    fill = fill + 1 == NS ? 0 : fill + 1;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int c = ks & 1, n = c ^ 1;
      if (ks + 1 < KS) {
#pragma unroll
        for (int i = 0; i < NI; ++i) a[n][i] = lda_(sc, fa[i], ks + 1);
#pragma unroll
        for (int j = 0; j < NJ; ++j) b[n][j] = lda_(sc, fb[j], ks + 1);
      } else {  // next stage's first fragments (published by the previous barrier)
#pragma unroll
        for (int i = 0; i < NI; ++i) a[n][i] = lda_(sn, fa[i], 0);
#pragma unroll
        for (int j = 0; j < NJ; ++j) b[n][j] = lda_(sn, fb[j], 0);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int m = 0; m < MF; ++m) {
        const int i = m / NJ, j = m % NJ;
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[c][i], b[c][j], acc[i][j], 0, 0, 0);
        if (m == 2 || m == 6) {
          __builtin_amdgcn_sched_barrier(0);
          issue(ks * 2 + (m == 6), sl);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
    // this wave's loads of stage st+2 have landed (those of stage st+3 may still be in flight); after the barrier
    // every wave's have, and every wave is done reading stage st
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"((D - 2) * LPS) : "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  big_epilogue<NJ, 64>(acc, ep, smem + (size_t)w * (NS * STAGE / NW), n0 + 128 * wm, k0 + 64 * wn, l, N, K);
}

// ---- A reduction-contiguous, B with the reduction index as its slow axis (the input gradient) -----------------
//   out[i][j] = sum over r of a[i][r] * b[r][j]        a: [I][R] (dz), b: [R][J] (w as stored), out: [I][J]
// The A side is gemm_dma_kernel's (64-byte tile rows, 16-byte fragment reads), the B side gemm_tn_kernel's
// ([32 reduction rows][256 columns] as in memory, transposing reads): no transposed copy of the weights is made.
// Needs R % 8 == 0.  A last stage of fewer than 32 reduction elements (R % 32 != 0) takes zeros for the missing rows
// of b; on the a side the lanes of the missing columns re-read the row's first chunk of that stage instead (inside
// the matrix, multiplied by zeros, and a non-finite value there belongs to the same output row anyway).
__global__ __launch_bounds__(512, 1) void gemm_nt_kernel(const bf16_t* __restrict__ A, int lda,
                                                         const bf16_t* __restrict__ Bm, int ldb, BigEpilogue ep, int I,
                                                         int J, int R, int tiles_i, int tiles_j, int splits,
                                                         float* __restrict__ part, int tail_first, int tail_splits) {
  constexpr int NW = 8, NI = 4, NJ = 2, KS = DK / 16, NS = 4, D = NS - 1;
  constexpr int ATILE = 256 * DROWB, BROWB = 512, BTILE = DK * BROWB, STAGE = ATILE + BTILE;  // 16 KB + 16 KB
  constexpr int QA = 2, QB = 2, LPS = QA + QB, MF = NI * NJ;
  __shared__ __attribute__((aligned(1024))) char smem[NS * STAGE];
  const int t = threadIdx.x, l = t & 63;
  const int w = __builtin_amdgcn_readfirstlane(t >> 6), wm = w >> 2, wn = w & 3;
  // splits > 1: the grid holds `splits` copies of the tile grid; copy z reduces its share of the stages and leaves an
  // fp32 partial product in part[z][I][J] (no bias, activation or rounding: the reducing kernel applies them)
  // tail_splits > 1 (with splits == 1): as in gemm_tn_kernel -- tiles [0, tail_first) are computed whole, each of the
  // others by tail_splits workgroups over shares of the reduction, which leave fp32 partial tiles in
  // part[z][tail tile][256][256] for nt_tail_store_kernel
  const int n_tiles = tiles_i * tiles_j;
  int z, bid, my_splits = splits, tail_tile = -1;
  if (tail_splits > 1 && (int)blockIdx.x >= tail_first) {
    const int e = (int)blockIdx.x - tail_first, r = n_tiles - tail_first;
    tail_tile = e % r;
    z = e / r;
    bid = tail_first + tail_tile;
    my_splits = tail_splits;
  } else {
    const int span = tail_splits > 1 ? tail_first : n_tiles;
    z = blockIdx.x / span;
    bid = blockIdx.x - z * span;
    const int per = span >> 3;
    if (bid < per * 8) bid = (bid & 7) * per + (bid >> 3);
  }
  int ti, tj;
  tn_tile_of(bid, tiles_i, tiles_j, ti, tj);
  const int i0 = ti * GM, j0 = tj * GN;
  int T = (R + DK - 1) / DK;
  const int tail = R % DK;          // reduction elements of a partial last stage (0: none)
  bool partial = tail != 0;         // this workgroup's last stage is that partial stage
  if (my_splits > 1) {
    const int s0 = (int)((long long)z * T / my_splits), s1 = (int)((long long)(z + 1) * T / my_splits);
    A += (size_t)s0 * DK;
    Bm += (size_t)s0 * DK * ldb;
    T = s1 - s0;
    partial = partial && z == my_splits - 1;
    ep.bias = nullptr; ep.mask = nullptr; ep.relu = 0; ep.out = nullptr; ep.upd_master = nullptr;
    if (tail_tile >= 0) {
      ep.out_f = part + ((size_t)z * (n_tiles - tail_first) + tail_tile) * (GM * GN) - ((ptrdiff_t)i0 * GN + j0);
      ep.ldo = GN;
    } else {
      ep.out_f = part + (size_t)z * I * J;
      ep.ldo = J;
    }
  }
  const bf16_t* const zero = reinterpret_cast<const bf16_t*>(g_tn_zero);

  uint32_t aoffs[QA];   // A: byte offset of this lane's chunk, rows clamped (they only feed outputs never stored)
  uint32_t aoffs_t[QA]; // the same for a partial last stage: chunks past the end re-read the stage's first chunk
#pragma unroll
  for (int q = 0; q < QA; ++q) {
    const int row = (q * NW + w) * 16 + (l >> 2), g = (l & 3) ^ dma_swz(row);
    const int ra = i0 + row < I ? i0 + row : I - 1;
    aoffs[q] = ((uint32_t)ra * (uint32_t)lda + g * 8) * 2u;
    aoffs_t[q] = ((uint32_t)ra * (uint32_t)lda + (g * 8 < tail ? g * 8 : 0)) * 2u;
  }
  const bf16_t* bp[QB];  // B: this lane's source for stage 0 (null: column outside the matrix)
  bool bcut[QB];         // this lane's row of a stage lies past the end of a partial last stage
#pragma unroll
  for (int q = 0; q < QB; ++q) {
    const int id = q * NW + w, r = 2 * id + (l >> 5);
    const int s16 = l & 31, blk = (s16 >> 2) ^ (r & 3);
    const int col = j0 + 32 * blk + 8 * (s16 & 3);
    bp[q] = col < J ? Bm + (size_t)r * ldb + col : nullptr;
    bcut[q] = r >= tail;
  }
  const size_t bstep = (size_t)DK * ldb;
  const uint32_t lds_base = lds_address_of(smem);
  int a_st = 0;  // reduction stage the next A loads fetch (clamped: the surplus is never read)
  int b_left[QB];  // stages the B loads have still to fetch
#pragma unroll
  for (int q = 0; q < QB; ++q) b_left[q] = T;
  auto issue = [&](int q, char* stage) {
    if (q < QA) {
      const int sidx = a_st < T ? a_st : T - 1;
      dma_load16_at(A + sidx * DK, (partial && sidx == T - 1) ? aoffs_t[q] : aoffs[q],
                    lds_base + (uint32_t)(stage - smem) + (uint32_t)((q * NW + w) * 1024));
      if (q == QA - 1) ++a_st;
    } else {
      // (B loads of stages past the end would read rows >= R of w: zeros instead)
      const int qb = q - QA;
      const bool live = b_left[qb] > 0;
      const bool cut = !live || bp[qb] == nullptr || (partial && b_left[qb] == 1 && bcut[qb]);
      dma_chunk64_at(cut ? zero : bp[qb], lds_base + (uint32_t)(stage - smem) + (uint32_t)(ATILE + (qb * NW + w) * 1024));
      if (live) {
        --b_left[qb];
        if (bp[qb] != nullptr) bp[qb] += bstep;
      }
    }
  };
  int fa[NI], fb[NJ];
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const int row = 128 * wm + 32 * i + (l & 31);
    fa[i] = row * DROWB + (((l >> 5) ^ dma_swz(row)) << 4);
  }
  const int mrow = 8 * (l >> 5) + ((l >> 2) & 3);
  const int chb = (16 * ((l >> 4) & 1) + 4 * (l & 3)) * 2;
#pragma unroll
  for (int j = 0; j < NJ; ++j) fb[j] = ATILE + mrow * BROWB + 64 * ((2 * wn + j) ^ (mrow & 3)) + chb;
  auto lda_ = [&](const char* stage, int o, int ks) { return frag(*reinterpret_cast<const uint4*>(stage + (o ^ (ks << 5)))); };
  auto ldb_ = [&](const char* stage, int o, int ks) { return tn_frag(stage + o + 16 * ks * BROWB, stage + o + (16 * ks + 4) * BROWB); };

  f32x16 acc[NI][NJ];
#pragma unroll
  for (int i = 0; i < NI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j) acc[i][j] = f32x16{0};
#pragma unroll
  for (int d = 0; d < D; ++d)
#pragma unroll
    for (int q = 0; q < LPS; ++q) issue(q, smem + d * STAGE);
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"((D - 2) * LPS) : "memory");
  __syncthreads();
  bf16x8 a[2][NI], b[2][NJ];
#pragma unroll
  for (int i = 0; i < NI; ++i) a[0][i] = lda_(smem, fa[i], 0);
#pragma unroll
  for (int j = 0; j < NJ; ++j) b[0][j] = ldb_(smem, fb[j], 0);
  int cur = 0, fill = D;
  for (int st = 0; st < T; ++st) {
    const char* sc = smem + cur * STAGE;
    cur = cur + 1 == NS ? 0 : cur + 1;
    const char* sn = smem + cur * STAGE;
    char* sl = smem + fill * STAGE;
    fill = fill + 1 == NS ? 0 : fill + 1;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int c = ks & 1, n = c ^ 1;
      const char* src = ks + 1 < KS ? sc : sn;  // next step's fragments; the next stage was published a barrier ago
      const int kn = ks + 1 < KS ? ks + 1 : 0;
#pragma unroll
      for (int i = 0; i < NI; ++i) a[n][i] = lda_(src, fa[i], kn);
#pragma unroll
      for (int j = 0; j < NJ; ++j) b[n][j] = ldb_(src, fb[j], kn);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int m = 0; m < MF; ++m) {
        const int i = m / NJ, j = m % NJ;
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[c][i], b[c][j], acc[i][j], 0, 0, 0);
        if (m == 2 || m == 6) {
          __builtin_amdgcn_sched_barrier(0);
          issue(ks * 2 + (m == 6), sl);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"((D - 2) * LPS) : "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  big_epilogue<NJ, 64>(acc, ep, smem + (size_t)w * (NS * STAGE / NW), i0 + 128 * wm, j0 + 64 * wn, l, I, J);
}

// column sums in two deterministic steps: partial sums over chunks of 128 rows, then the chunks in order
constexpr int kColsumRows = 128;
__global__ __launch_bounds__(256) void colsum_partial_kernel(const bf16_t* __restrict__ z, float* __restrict__ part,
                                                             int M, int N) {
  const int n = blockIdx.x * blockDim.x + threadIdx.x;
  if (n >= N) return;
  const int m0 = blockIdx.y * kColsumRows, m1 = m0 + kColsumRows < M ? m0 + kColsumRows : M;
  float s = 0.f;
  for (int m = m0; m < m1; ++m) s += bf2f(z[(size_t)m * N + n]);
  part[(size_t)blockIdx.y * N + n] = s;
}
// The same with eight columns per thread (16-byte loads) and the loads of eight rows issued before their adds; per
// column the rows are still added in ascending order.  N % 8 == 0, z 16-byte aligned.
__global__ __launch_bounds__(256) void colsum_partial8_kernel(const bf16_t* __restrict__ z, float* __restrict__ part,
                                                              int M, int N) {
  const int n = (blockIdx.x * blockDim.x + threadIdx.x) * 8;
  if (n >= N) return;
  const int m0 = blockIdx.y * kColsumRows, m1 = m0 + kColsumRows < M ? m0 + kColsumRows : M;
  float s[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  constexpr int kBatch = 8;
  for (int mb = m0; mb < m1; mb += kBatch) {
    uint4 v[kBatch];
#pragma unroll
    for (int q = 0; q < kBatch; ++q) {
      const int m = mb + q < m1 ? mb + q : m1 - 1;  // past the end: a valid row, dropped below
      v[q] = ldg16(z + (size_t)m * N + n);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int q = 0; q < kBatch; ++q) {
      uint16_t h[8];
      unpack8(v[q], h);
      const bool on = mb + q < m1;
#pragma unroll
      for (int c = 0; c < 8; ++c) s[c] = on ? s[c] + bf2f(h[c]) : s[c];
    }
  }
  float* o = part + (size_t)blockIdx.y * N + n;
  *reinterpret_cast<float4*>(o) = make_float4(s[0], s[1], s[2], s[3]);
  *reinterpret_cast<float4*>(o + 4) = make_float4(s[4], s[5], s[6], s[7]);
}
__global__ __launch_bounds__(256) void colsum_final_kernel(const float* __restrict__ part, float* __restrict__ out,
                                                           int chunks, int N) {
  const int n = blockIdx.x * blockDim.x + threadIdx.x;
  if (n >= N) return;
  float s = 0.f;
  for (int c = 0; c < chunks; ++c) s += part[(size_t)c * N + n];
  out[n] = s;
}

void launch_colsum_partial(hipStream_t s, const bf16_t* z, float* part, int M, int N, int chunks) {
  if ((N % 8) == 0 && ((reinterpret_cast<uintptr_t>(z) | reinterpret_cast<uintptr_t>(part)) & 15) == 0)
    colsum_partial8_kernel<<<dim3((N / 8 + 255) / 256, chunks), 256, 0, s>>>(z, part, M, N);
  else
    colsum_partial_kernel<<<dim3((N + 255) / 256, chunks), 256, 0, s>>>(z, part, M, N);
}

__global__ __launch_bounds__(256) void colsum_kernel(const bf16_t* __restrict__ z, float* __restrict__ out, int M,
                                                     int N) {
  const int n = blockIdx.x * blockDim.x + threadIdx.x;
  if (n >= N) return;
  float s = 0.f;
  for (int m = 0; m < M; ++m) s += bf2f(z[(size_t)m * N + n]);
  out[n] = s;
}

// Variant of the forward product.  Measured at 8192 x 4096 (MI355X, % of the nominal bf16 peak): reduction 25088 --
// 64-byte rows, 8 waves 44-48; 128-byte rows, 8 waves 49-53; 128-byte rows, 4 waves 55-56.  Reduction 4096 -- 46-48;
// 48-50; 45.  Hence four waves from a reduction length of 8192 on.
int g_big_waves = 0;        // 0: by reduction length; 4 or 8: forced
int g_big_row_bytes = 128;  // LDS tile rows of the forward product: 128 (64 reduction elements per stage) or 64
constexpr int kFourWaveMinR = 8192;
bool g_wgrad_tn = true;

// splits > 1 (with `part`, splits * I * J floats): only the 128-byte-row forward kernel can split its reduction;
// hipErrorInvalidValue if the shape does not let it run.
template <bool TA, bool TB>
hipError_t launch_big(hipStream_t s, const bf16_t* a, int lda, const bf16_t* b, int ldb, const BigEpilogue& ep, int I,
                      int J, int R, int splits = 1, float* part = nullptr) {
  dim3 grid((J + GN - 1) / GN, (I + GM - 1) / GM);
  if (!TA && !TB && R >= DK && (R % 8) == 0 && (lda % 8) == 0 && (ldb % 8) == 0 &&
      ((reinterpret_cast<uintptr_t>(a) | reinterpret_cast<uintptr_t>(b)) & 15) == 0 &&
      (size_t)I * lda < ((size_t)1 << 31) && (size_t)J * ldb < ((size_t)1 << 31)) {  // 32-bit byte offsets
    const bool wide_rows = (g_big_row_bytes == 128 || splits > 1) && (R % EK) == 0 && R >= 2 * EK * splits;
    if (splits > 1 && !wide_rows) return hipErrorInvalidValue;
    // four waves (one per SIMD) pay off when the reduction is long enough to amortise their slower start and end
    const int waves = g_big_waves ? g_big_waves : ((wide_rows && R / splits >= kFourWaveMinR) ? 4 : 8);
    const unsigned n = grid.x * grid.y * (unsigned)splits;
    const int ty = (int)grid.y, tx = (int)grid.x;
    if (wide_rows && waves == 4) gemm_dma64_kernel<4><<<n, 256, 0, s>>>(a, lda, b, ldb, ep, I, J, R, ty, tx, splits, part);
    else if (wide_rows) gemm_dma64_kernel<8><<<n, 512, 0, s>>>(a, lda, b, ldb, ep, I, J, R, ty, tx, splits, part);
    else if (waves == 4) gemm_dma_kernel<4><<<n, 256, 0, s>>>(a, lda, b, ldb, ep, I, J, R, ty, tx);
    else gemm_dma_kernel<8><<<n, 512, 0, s>>>(a, lda, b, ldb, ep, I, J, R, ty, tx);
    return hipGetLastError();
  }
  if (splits > 1) return hipErrorInvalidValue;
  if (g_big_waves != 4) gemm_big_kernel<TA, TB, 8><<<grid, 512, 0, s>>>(a, lda, b, ldb, ep, I, J, R);
  else gemm_big_kernel<TA, TB, 4><<<grid, 256, 0, s>>>(a, lda, b, ldb, ep, I, J, R);
  return hipGetLastError();
}

}  // namespace

int set_big_gemm_waves(int waves) {
  const int old = g_big_waves + (g_big_row_bytes == 64 ? 100 : 0);
  switch (waves) {
    case 0: case 4: case 8: g_big_waves = waves; g_big_row_bytes = 128; break;
    case 104: case 108: g_big_waves = waves - 100; g_big_row_bytes = 64; break;
    default: break;
  }
  return old;
}

hipError_t linear_fwd_big_bf16(hipStream_t s, const bf16_t* x, int ldx, const bf16_t* w, const bf16_t* b, bf16_t* y,
                               float* y_f32, int M, int N, int K, bool relu, int splits, float* part) {
  BigEpilogue ep = {b, nullptr, relu ? 1 : 0, y, y_f32, N};
  return launch_big<false, false>(s, x, ldx, w, K, ep, M, N, K, splits, part);
}

// Operands stored sideways go through a transposing pre-pass when the caller provides scratch: the 2x8-block
// transposing LDS stores cost more issue slots than the MFMAs of a stage, while a separate transpose is a small
// streaming kernel (measured: 12 % -> about 30 % of MFMA peak for the weight gradient at 8192 rows).
size_t linear_dgrad_big_scratch_bytes(int N, int K) { return (size_t)N * K * sizeof(bf16_t); }
size_t linear_wgrad_big_scratch_bytes(int M, int N, int K) { return (size_t)M * ((size_t)N + K) * sizeof(bf16_t); }

// A weight gradient with too few 256 x 256 tiles for the chip and many rows: the rows are split this many ways
// (one workgroup per compute unit or so, at least 8 stages of 32 rows each); 1 = no split.  S2VT's recurrent
// matrices (4000 x 1000 outputs, 5120 rows) are 64 tiles: 154 us on 64 compute units.
static int wgrad_big_splits(int M, int N, int K) {
  const int tiles = ((N + GM - 1) / GM) * ((K + GN - 1) / GN);
  if (tiles >= 128 || (N % 4) != 0 || (K % 4) != 0 || (((size_t)N * K) % 4) != 0) return 1;
  int sp = 256 / tiles;
  if (sp > M / 256) sp = M / 256;
  if (sp > 16) sp = 16;
  return sp >= 2 ? sp : 1;
}
// A weight gradient whose tile count is a little over a multiple of the compute units: the tiles of the last,
// partly filled round have their rows split so that the round takes a fraction of a tile's time (gemm_tn_kernel's
// tail_first / tail_splits).  first: tiles computed whole; tiles: tiles of the tail; splits: workgroups per tail tile.
struct TailPlan {
  int first, tiles, splits;
  size_t bytes;
};
static int device_compute_units() {
  int dev = 0, n = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
    return 0;
  return n;
}
static bool tail_plan(int tiles, int max_splits, TailPlan& p) {
  const int cus = device_compute_units();
  if (cus < 8 || (cus % 8) != 0 || tiles < cus) return false;
  const int r = tiles % cus;
  if (r == 0 || 2 * r > cus) return false;
  int sp = cus / r;
  if (sp > max_splits) sp = max_splits;
  if (sp > 16) sp = 16;
  if (sp < 2) return false;
  p.first = tiles - r;  // (a multiple of 8: the renumbering over the XCDs covers all of it)
  p.tiles = r;
  p.splits = sp;
  p.bytes = (size_t)sp * r * GM * GN * sizeof(float);
  return true;
}
static bool wgrad_tail_plan(int M, int N, int K, TailPlan& p) {
  if (M < 512 || (N % 8) != 0 || (K % 8) != 0) return false;
  return tail_plan(((N + GM - 1) / GM) * ((K + GN - 1) / GN), M / 256, p);
}
size_t linear_wgrad_update_big_scratch_bytes(int M, int N, int K) {
  const int sp = wgrad_big_splits(M, N, K);
  if (sp > 1) return (size_t)sp * N * K * sizeof(float);
  TailPlan tp;
  return wgrad_tail_plan(M, N, K, tp) ? tp.bytes : 0;
}

// splits > 1: the reduction (over the N out-features) is split; `scratch` then receives splits * M * K floats of
// partial products instead of serving as room for transposed weights, and mask / dx are not touched (the reducing
// kernel applies them); hipErrorInvalidValue if the shape does not allow the kernel that can do that.
hipError_t linear_dgrad_big_bf16(hipStream_t s, const bf16_t* dz, const bf16_t* w, const bf16_t* mask, bf16_t* dx, int M,
                                 int N, int K, void* scratch, size_t scratch_bytes, int splits) {
  BigEpilogue ep = {nullptr, mask, 0, dx, nullptr, K};
  if (g_wgrad_tn && (N % 8) == 0 && (K % 8) == 0 && ((reinterpret_cast<uintptr_t>(dz) | reinterpret_cast<uintptr_t>(w)) & 15) == 0 &&
      (size_t)M * N < ((size_t)1 << 31) && N / DK >= 4 * splits) {  // w as stored: transposing LDS reads on the B side
    const int ti = (M + GM - 1) / GM, tj = (K + GN - 1) / GN;
    if (splits > 1 && (!scratch || scratch_bytes < (size_t)splits * M * K * sizeof(float))) return hipErrorInvalidValue;
    TailPlan tp;
    if (splits == 1 && dx && tail_plan(ti * tj, N / DK / 8, tp) && scratch && scratch_bytes >= tp.bytes &&
        (reinterpret_cast<uintptr_t>(scratch) & 15) == 0 && (reinterpret_cast<uintptr_t>(dx) & 7) == 0 &&
        (!mask || (reinterpret_cast<uintptr_t>(mask) & 7) == 0)) {
      float* parts = static_cast<float*>(scratch);
      gemm_nt_kernel<<<tp.first + tp.tiles * tp.splits, 512, 0, s>>>(dz, N, w, K, ep, M, K, N, ti, tj, 1, parts, tp.first,
                                                                      tp.splits);
      hipError_t e = hipGetLastError();
      if (e != hipSuccess) return e;
      nt_tail_store_kernel<<<tp.tiles * 64, 256, 0, s>>>(parts, tp.tiles, tp.splits, tp.first, ti, tj, M, K, mask, dx);
      return hipGetLastError();
    }
    gemm_nt_kernel<<<ti * tj * splits, 512, 0, s>>>(dz, N, w, K, ep, M, K, N, ti, tj, splits, static_cast<float*>(scratch), 0, 0);
    return hipGetLastError();
  }
  if (splits > 1) return hipErrorInvalidValue;
  if (scratch && M >= 2048 && scratch_bytes >= linear_dgrad_big_scratch_bytes(N, K)) {  // worth a pass over w
    bf16_t* wt = static_cast<bf16_t*>(scratch);  // [K][N]
    hipError_t e = transpose_bf16(s, w, wt, N, K);
    if (e != hipSuccess) return e;
    return launch_big<false, false>(s, dz, N, wt, N, ep, M, K, N);
  }
  return launch_big<false, true>(s, dz, N, w, K, ep, M, K, N);
}

hipError_t linear_wgrad_big_bf16(hipStream_t s, const bf16_t* dz, const bf16_t* x, float* dw, float* db, int M, int N,
                                 int K, void* scratch, size_t scratch_bytes) {
  BigEpilogue ep = {nullptr, nullptr, 0, nullptr, dw, K};
  hipError_t e;
  const int chunks = (M + kColsumRows - 1) / kColsumRows;
  bool db_done = false;
  if (db && scratch && scratch_bytes >= (size_t)chunks * N * sizeof(float)) {  // before the scratch is reused below
    float* cp = static_cast<float*>(scratch);
    launch_colsum_partial(s, dz, cp, M, N, chunks);
    colsum_final_kernel<<<(N + 255) / 256, 256, 0, s>>>(cp, db, chunks, N);
    db_done = true;
  }
  if (g_wgrad_tn && (N % 8) == 0 && (K % 8) == 0 &&
      ((reinterpret_cast<uintptr_t>(dz) | reinterpret_cast<uintptr_t>(x)) & 15) == 0) {
    // operands as they are: transposing LDS reads instead of a transposing pre-pass
    const int tn = (N + GM - 1) / GM, tk = (K + GN - 1) / GN;
    gemm_tn_kernel<<<tn * tk, 512, 0, s>>>(dz, N, x, K, ep, M, N, K, tn, tk, 1, nullptr, 0, 0);
    e = hipGetLastError();
  } else if (scratch && (M % 8) == 0 && scratch_bytes >= linear_wgrad_big_scratch_bytes(M, N, K)) {
    bf16_t* zt = static_cast<bf16_t*>(scratch);  // [N][M]
    bf16_t* xt = zt + (size_t)N * M;             // [K][M]
    e = transpose_bf16(s, dz, zt, M, N);
    if (e == hipSuccess) e = transpose_bf16(s, x, xt, M, K);
    if (e == hipSuccess) e = launch_big<false, false>(s, zt, M, xt, M, ep, N, K, M);
  } else {
    e = launch_big<true, true>(s, dz, N, x, K, ep, N, K, M);
  }
  if (e != hipSuccess) return e;
  if (db && !db_done) colsum_kernel<<<(N + 255) / 256, 256, 0, s>>>(dz, db, M, N);
  return hipGetLastError();
}


// g = dz^T x fused with the momentum-SGD step (see BigEpilogue) when the transposing-read kernel applies; otherwise
// g goes to `part` (N*K + N floats) and the separate reduce + update kernel applies the step.  The bias uses the
// column sums of dz either way.  part may be null only if the fused kernel is known to apply.
hipError_t linear_wgrad_update_big_bf16(hipStream_t s, const bf16_t* dz, const bf16_t* x, float* part, int M, int N,
                                        int K, float* master_w, float* mom_w, bf16_t* ring_w, float* master_b,
                                        float* mom_b, bf16_t* ring_b, UpdateRule rule, void* scratch,
                                        size_t scratch_bytes) {
  const size_t n_w = (size_t)N * K;
  const bool fused = g_wgrad_tn && (N % 8) == 0 && (K % 8) == 0 &&
                     ((reinterpret_cast<uintptr_t>(dz) | reinterpret_cast<uintptr_t>(x) |
                       reinterpret_cast<uintptr_t>(master_w) | reinterpret_cast<uintptr_t>(mom_w)) & 15) == 0 &&
                     (reinterpret_cast<uintptr_t>(ring_w) & 7) == 0;
  if (!fused) {
    if (!part) return hipErrorInvalidValue;
    hipError_t e = linear_wgrad_big_bf16(s, dz, x, part, master_b ? part + n_w : nullptr, M, N, K, scratch, scratch_bytes);
    if (e != hipSuccess) return e;
    return wgrad_reduce_update(s, part, 1, 0, n_w, master_b ? N : 0, master_w, mom_w, ring_w, master_b, mom_b, ring_b, rule);
  }
  if (master_b) {  // bias first: its column sums use the scratch
    if (!part) return hipErrorInvalidValue;
    float* db = part + n_w;
    const int chunks = (M + kColsumRows - 1) / kColsumRows;
    if (scratch && scratch_bytes >= (size_t)chunks * N * sizeof(float)) {
      float* cp = static_cast<float*>(scratch);
      launch_colsum_partial(s, dz, cp, M, N, chunks);
      colsum_final_kernel<<<(N + 255) / 256, 256, 0, s>>>(cp, db, chunks, N);
    } else {
      colsum_kernel<<<(N + 255) / 256, 256, 0, s>>>(dz, db, M, N);
    }
    hipError_t e = wgrad_reduce_update(s, db, 1, 0, 0, N, nullptr, nullptr, nullptr, master_b, mom_b, ring_b, rule);
    if (e != hipSuccess) return e;
  }
  BigEpilogue ep = {nullptr, nullptr, 0, nullptr, nullptr, K, master_w, mom_w, ring_w, rule};
  const int tn = (N + GM - 1) / GM, tk = (K + GN - 1) / GN;
  const int sp = wgrad_big_splits(M, N, K);
  if (sp > 1 && scratch && scratch_bytes >= (size_t)sp * n_w * sizeof(float)) {
    float* parts = static_cast<float*>(scratch);  // (the column sums above are done with it: same stream)
    gemm_tn_kernel<<<tn * tk * sp, 512, 0, s>>>(dz, N, x, K, ep, M, N, K, tn, tk, sp, parts, 0, 0);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return wgrad_reduce_update(s, parts, sp, n_w, n_w, 0, master_w, mom_w, ring_w, nullptr, nullptr, nullptr, rule);
  }
  TailPlan tp;
  if (wgrad_tail_plan(M, N, K, tp) && scratch && scratch_bytes >= tp.bytes &&
      (reinterpret_cast<uintptr_t>(scratch) & 15) == 0) {
    float* parts = static_cast<float*>(scratch);
    gemm_tn_kernel<<<tp.first + tp.tiles * tp.splits, 512, 0, s>>>(dz, N, x, K, ep, M, N, K, tn, tk, 1, parts, tp.first,
                                                                    tp.splits);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    tn_tail_update_kernel<<<tp.tiles * 64, 256, 0, s>>>(parts, tp.tiles, tp.splits, tp.first, tn, tk, N, K, master_w,
                                                        mom_w, ring_w, rule);
    return hipGetLastError();
  }
  gemm_tn_kernel<<<tn * tk, 512, 0, s>>>(dz, N, x, K, ep, M, N, K, tn, tk, 1, nullptr, 0, 0);
  return hipGetLastError();
}

}  // namespace pd
