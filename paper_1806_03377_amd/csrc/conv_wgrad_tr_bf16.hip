// Weight gradient of a stride-1 bf16 convolution with at most "same" padding (NHWC, fp32 accumulate) for gfx950:
//   dW[co][ta][tb][ci] = sum over output pixels p of dz[p][co] * x[p shifted by tap (ta, tb)][ci]
// as partial sums over ranges of pixels (the caller adds the partials in a fixed order and applies the update).
//
// Both operands have the reduction index (the pixel) as their slow axis in memory.  Instead of transposing them
// in registers, tiles go into LDS as they lie in memory ([pixel][channel], straight from global memory with
// global_load_lds) and the MFMA operands are fetched with the transposing LDS read (ds_read_b64_tr_b16): within a
// group of 16 lanes, source lane j supplies the address of 4 channels (j % 4) of pixel (j / 4), and lane i
// receives channel i of those 4 pixels -- exactly a "row i, 4 reduction elements" piece of a 32x32x16 operand.
//
// All taps of a group of filter rows are accumulated by ONE workgroup, so dz is read once instead of once per
// tap.  To make every tap a constant shift of the input, pixels are numbered in a padded row-major space
// ("virtual pixels"): rows have Wp = W + pw positions, position u of a row is input column u - pw (u < pw is the
// zero padding, which the end of a row shares with the beginning of the next) and output column u (u >= Wo: no
// output, dz is read as zero; likewise the last H - Ho rows of every image when the layer is padded less than
// "same": pixels are numbered by input rows, a dz row is found from the count of output-less rows before it).  Tap (ta, tb) of output pixel v is then input position v + (ta - ph) Wp + tb.
// A stage holds 64 virtual pixels: a [64][COT] tile of dz and, per filter row of the group, a band of
// 64 + kw - 1 consecutive input positions x 64 input channels.  Whatever falls into the padding, outside the
// image or beyond the last channel is fetched from a 16-byte block of zeros, so the inner loop has no masks.
//
// A wave accumulates AI x 32 output channels x 32 input channels x all taps of the group: AI = 2 (four waves per
// workgroup, one per SIMD) while that is at most 16 accumulator tiles, the capacity of the accumulation
// registers; AI = 1 (eight waves, two per SIMD) for the nine taps of a 3x3 filter.  COT = 128: the waves tile
// 128 co x 64 ci.  COT = 64 (layers with <= 64 output channels): 64 co x 64 ci x the two halves of the stage's
// pixels, and the two pixel halves write separate partial sums.
// Three stages in LDS; the loads of stage n+2 are spread between the MFMAs of stage n.
#include "bf16_util.h"
#include "mfma_util.h"
#include "pd_kernels.h"

namespace pd {
namespace {

__device__ __attribute__((aligned(16))) const uint32_t g_zero_block[4] = {0u, 0u, 0u, 0u};
typedef __attribute__((address_space(3))) void lds_void_t;
typedef short v4i16_t __attribute__((ext_vector_type(4)));
typedef short v8i16_t __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) v4i16_t lds_v4i16_t;
typedef __attribute__((address_space(3))) char lds_char_t;

#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
// one 16-byte chunk per lane, global -> LDS: lane L's chunk lands at uniform_lds_dst + 16 L
__device__ __forceinline__ void dma_chunk(const bf16_t* lane_src, lds_char_t* uniform_lds_dst) {
  const uint32_t lds_addr = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)uniform_lds_dst);
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(lane_src), "s"(lds_addr) : "memory", "m0");
}
#pragma clang diagnostic pop

// 16-byte MFMA operand from two transposing reads (reduction elements 0..3 and 4..7 of this lane's row)
__device__ __forceinline__ bf16x8 tr_frag(const lds_char_t* lo, const lds_char_t* hi) {
  const v4i16_t a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16_t*)lo);
  const v4i16_t b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16_t*)hi);
  const v8i16_t v = __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, v);
}

constexpr int kPix = 64;    // virtual pixels per stage
constexpr int kXRow = 128;  // bytes of one input position in LDS: 64 input channels

template <int GR, int KW, int COT, int AI>
__global__ __launch_bounds__(512 / AI, 1) void conv_wgrad_tr_kernel(const bf16_t* __restrict__ dZ,
                                                               const bf16_t* __restrict__ X, float* __restrict__ part,
                                                               ConvGeom g, int chunks_per_split, int tap_groups) {
  constexpr int NT = GR * KW;                        // taps accumulated by this workgroup
  constexpr int ZRB = COT * 2;                       // bytes of one pixel of the dz tile
  constexpr int ZT = kPix * ZRB;                     // dz tile
  constexpr int XG = (kPix + KW - 1 + 7) / 8;        // groups of 8 input positions per band
  constexpr int XB = XG * 8 * kXRow;                 // one band
  constexpr int STAGE = ZT + GR * XB;
  constexpr int NS = 3;
  constexpr int NWV = 8 / AI;                        // waves
  constexpr int NZL = ZT / 1024, NXL = GR * XG;      // wave-wide loads per stage
  constexpr int ZPW = NZL / NWV, XPW = (NXL + NWV - 1) / NWV;  // per wave (surplus x loads repeat the last one)
  constexpr int LPS = ZPW + XPW;
  constexpr int KSW = COT == 128 ? 4 : 2;            // 16-pixel reduction steps per wave and stage
  constexpr int MFS = KSW * AI * NT;                 // MFMAs per wave and stage
  static_assert(NZL % NWV == 0, "dz loads divide evenly");
  constexpr int GAP = MFS / LPS > 0 ? MFS / LPS : 1;
  static_assert(NS * STAGE <= 160 * 1024, "LDS");
  static_assert(MFS >= LPS, "every load needs an MFMA to hide behind");
  __shared__ __attribute__((aligned(1024))) char smem_[NS * STAGE];
  lds_char_t* const smem = (lds_char_t*)smem_;

  const int t = threadIdx.x, l = t & 63;
  const int w = __builtin_amdgcn_readfirstlane(t >> 6), wc = w & 1;
  // COT = 128: the other wave bits select the wave's output-channel blocks; COT = 64: also the pixel half
  constexpr int WCO = (COT / 32) / AI;               // waves along the output channels
  const int wrow = (w >> 1) % WCO, wh = (w >> 1) / WCO;
  const int cb0 = AI * wrow;                         // first 32-channel block of this wave inside the co tile
  const int taps = g.kh * g.kw;
  const int ci_tiles = (g.Ci + 63) / 64;
  // Workgroups are dealt round-robin to the 8 XCDs (each with its own L2): renumber them so that all tiles of a
  // pixel range -- they read the same dz and x -- run on the same XCD, one range after the other.
  int tile_id, split_id;
  {
    const int tiles = gridDim.x, total = tiles * gridDim.y, per = total >> 3;
    int id = blockIdx.x + tiles * blockIdx.y;
    if (id < per * 8) id = (id & 7) * per + (id >> 3);
    split_id = id / tiles;
    tile_id = id - split_id * tiles;
  }
  const int tg = tile_id % tap_groups;
  const int ci0 = ((tile_id / tap_groups) % ci_tiles) * 64;
  const int co0 = (tile_id / tap_groups / ci_tiles) * COT;
  const int ta0 = tg * GR;
  const int Wp = g.W + g.pw, NH = g.N * g.H;
  const int nchunks = (NH * Wp + kPix - 1) / kPix;
  const int chunk0 = split_id * chunks_per_split;
  const int chunk1 = chunk0 + chunks_per_split < nchunks ? chunk0 + chunks_per_split : nchunks;
  const int q64 = kPix / Wp, r64 = kPix - q64 * Wp, qH = q64 % g.H;
  const bf16_t* const zero = reinterpret_cast<const bf16_t*>(g_zero_block);

  // ---- loader state: every lane owns one 16-byte chunk of ZPW dz loads and XPW x loads per stage -----------
  // (an unpadded or partly padded layer has fewer output rows and columns than input ones: dH input rows of every
  // image and the last W - Wo positions of every row carry no output)
  const int dH = g.H - g.Ho, qN = q64 / g.H;
  int zR[ZPW], zu[ZPW], zc[ZPW];  // padded row index, position in the row, first output channel (-1: none)
  int zh[ZPW], zskip[ZPW];        // row inside its image; rows without output in the images before it
#pragma unroll
  for (int i = 0; i < ZPW; ++i) {
    const int q = w + NWV * i;
    int row, b, piece;
    if (COT == 128) {
      row = 4 * q + (l >> 4);
      piece = l & 3;
      b = ((l >> 2) & 3) ^ (row & 3);
    } else {
      row = 8 * q + (l >> 3);
      piece = l & 3;
      b = ((l >> 2) & 1) ^ ((row >> 1) & 1);
    }
    const int v = chunk0 * kPix + row;
    zR[i] = v / Wp;
    zu[i] = v - zR[i] * Wp;
    zh[i] = zR[i] % g.H;
    zskip[i] = (zR[i] / g.H) * dH;
    const int co = co0 + 32 * b + 8 * piece;
    zc[i] = co < g.Co ? co : -1;
  }
  int xR[XPW], xh[XPW], xu[XPW], xc[XPW], xdt[XPW], xdst[XPW];
#pragma unroll
  for (int i = 0; i < XPW; ++i) {
    int q = w + NWV * i;
    if (q > NXL - 1) q = NXL - 1;
    const int band = q / XG, grp = q - band * XG;
    const int row = 8 * grp + (l >> 3);
    const int b = ((l >> 2) & 1) ^ ((row >> 1) & 1);
    const int v = chunk0 * kPix + row;
    xR[i] = v / Wp;
    xu[i] = v - xR[i] * Wp;
    xh[i] = xR[i] % g.H;
    const int ci = ci0 + 32 * b + 8 * (l & 3);
    xc[i] = (ci < g.Ci && ta0 + band < g.kh) ? ci : -1;
    xdt[i] = ta0 + band - g.ph;
    xdst[i] = ZT + band * XB + grp * 1024;
  }
  auto issue = [&](int q, lds_char_t* stage) {  // q-th load of this wave for the next stage; advances by one stage
    // (addresses are formed unconditionally and selected afterwards: no branches around the loads)
    if (q < ZPW) {
      const int i = q;
      const bool ok = zc[i] >= 0 && zR[i] < NH && zu[i] < g.Wo && zh[i] < g.Ho;
      const bf16_t* cand = dZ + ((long long)((zR[i] - zskip[i]) * g.Wo + zu[i]) * g.Co + zc[i]);
      dma_chunk(ok ? cand : zero, stage + (w + NWV * i) * 1024);
      zu[i] += r64;
      zR[i] += q64;
      const int carry = zu[i] >= Wp ? 1 : 0;
      zu[i] -= carry ? Wp : 0;
      zR[i] += carry;
      zh[i] += qH + carry;
      const int wrap = zh[i] >= g.H ? 1 : 0;
      zh[i] -= wrap ? g.H : 0;
      zskip[i] += (qN + wrap) * dH;
    } else {
      const int i = q - ZPW;
      const int hi = xh[i] + xdt[i];
      const bool ok = xc[i] >= 0 && xu[i] >= g.pw && xR[i] < NH && (unsigned)hi < (unsigned)g.H;
      const bf16_t* cand = X + ((long long)((xR[i] + xdt[i]) * g.W + (xu[i] - g.pw)) * g.Ci + xc[i]);
      dma_chunk(ok ? cand : zero, stage + xdst[i]);
      xu[i] += r64;
      xR[i] += q64;
      xh[i] += qH;  // only the row inside its image matters: advance modulo H
      const int carry = xu[i] >= Wp ? 1 : 0;
      xu[i] -= carry ? Wp : 0;
      xR[i] += carry;
      xh[i] += carry;
      xh[i] -= xh[i] >= g.H ? g.H : 0;
    }
  };

  // ---- fragment addresses (bytes inside a stage) for reduction step 0, low half ---------------------------
  const int pixl = 8 * (l >> 5) + ((l >> 2) & 3);
  const int chb = (16 * ((l >> 4) & 1) + 4 * (l & 3)) * 2;
  int aoff[AI], boff0;
#pragma unroll
  for (int i = 0; i < AI; ++i) {
    if (COT == 128) aoff[i] = pixl * ZRB + 64 * ((cb0 + i) ^ (pixl & 3)) + chb;
    else aoff[i] = (32 * wh + pixl) * ZRB + 64 * ((cb0 + i) ^ ((pixl >> 1) & 1)) + chb;
  }
  {
    const int j = (COT == 128 ? 0 : 32 * wh) + pixl;
    boff0 = ZT + j * kXRow + 64 * (wc ^ ((j >> 1) & 1)) + chb;
  }

  f32x16 acc[AI][NT], accb[AI];
#pragma unroll
  for (int i = 0; i < AI; ++i) {
    accb[i] = f32x16{0};
#pragma unroll
    for (int n = 0; n < NT; ++n) acc[i][n] = f32x16{0};
  }
  const bool do_bias = tg == 0 && ci0 == 0 && wc == 0;  // wave-uniform
  const bf16x8 ones = __builtin_bit_cast(bf16x8, make_uint4(0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u));

  if (chunk0 < chunk1) {
#pragma unroll
    for (int d = 0; d < 2; ++d)
#pragma unroll
      for (int q = 0; q < LPS; ++q) issue(q, smem + d * STAGE);
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LPS) : "memory");  // stage 0 has landed
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    int cur = 0, fill = 2;
    for (int ch = chunk0; ch < chunk1; ++ch) {
      const lds_char_t* sc = smem + cur * STAGE;
      cur = cur == NS - 1 ? 0 : cur + 1;
      lds_char_t* sl = smem + fill * STAGE;
      fill = fill == NS - 1 ? 0 : fill + 1;
      // The KW taps of a filter row read overlapping windows of the same band: this lane's 8 + KW - 1 consecutive
      // input positions are fetched once (NR transposing reads of 4 positions each) and every tap's operand is cut
      // out of that window in registers.  The windows are software-pipelined by hand: the reads of row r + 2 (two
      // filter rows ahead, across reduction steps) are issued, and pinned, before the MFMAs of row r, so that the
      // LDS latency is covered by two rows of MFMAs.
      constexpr int NR = (KW + 7 + 3) / 4, ROWS = KSW * GR, PF = 2;
      uint32_t wv[PF + 1][2 * NR];
      bf16x8 a[PF + 1][AI];  // (a row at most PF ahead is at most PF reduction steps ahead)
      auto read_row = [&](int r, int buf) {
        const int ks = r / GR, ta = r % GR;
        const int za = 16 * ks * ZRB, xa = 16 * ks * kXRow;
        if (ta == 0) {
#pragma unroll
          for (int i = 0; i < AI; ++i) a[ks % (PF + 1)][i] = tr_frag(sc + aoff[i] + za, sc + aoff[i] + za + 4 * ZRB);
        }
#pragma unroll
        for (int h = 0; h < NR; ++h) {
          const v4i16_t rr = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16_t*)(sc + boff0 + ta * XB + xa + 4 * h * kXRow));
          const uint2 rw = __builtin_bit_cast(uint2, rr);
          wv[buf][2 * h] = rw.x;
          wv[buf][2 * h + 1] = rw.y;
        }
      };
#pragma unroll
      for (int r = 0; r < PF && r < ROWS; ++r) read_row(r, r);
#pragma unroll
      for (int r = 0; r < ROWS; ++r) {
        const int ks = r / GR, ta = r % GR, cb = r % (PF + 1);
        if (r + PF < ROWS) read_row(r + PF, (r + PF) % (PF + 1));
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int tb = 0; tb < KW; ++tb) {
          const int n = ta * KW + tb;
          uint4 o;
          if (tb % 2 == 0) {
            o = make_uint4(wv[cb][tb / 2], wv[cb][tb / 2 + 1], wv[cb][tb / 2 + 2], wv[cb][tb / 2 + 3]);
          } else {
            const int q = (tb - 1) / 2;
            o = make_uint4(__builtin_amdgcn_alignbit(wv[cb][q + 1], wv[cb][q], 16),
                           __builtin_amdgcn_alignbit(wv[cb][q + 2], wv[cb][q + 1], 16),
                           __builtin_amdgcn_alignbit(wv[cb][q + 3], wv[cb][q + 2], 16),
                           __builtin_amdgcn_alignbit(wv[cb][q + 4], wv[cb][q + 3], 16));
          }
          const bf16x8 b = frag(o);
#pragma unroll
          for (int i = 0; i < AI; ++i) {
            acc[i][n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks % (PF + 1)][i], b, acc[i][n], 0, 0, 0);
            const int m = (ks * NT + n) * AI + i;
            if (m % GAP == GAP - 1 && m / GAP < LPS) {
              __builtin_amdgcn_sched_barrier(0);
              issue(m / GAP, sl);
              __builtin_amdgcn_sched_barrier(0);
            }
          }
        }
        if (do_bias && ta == GR - 1) {
#pragma unroll
          for (int i = 0; i < AI; ++i)
            accb[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks % (PF + 1)][i], ones, accb[i], 0, 0, 0);
        }
      }
      // this wave's loads of the next stage have landed (those of the one after may be in flight); after the
      // barrier every wave's have, and every wave is done reading the current stage
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LPS) : "memory");
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  }

  const size_t n_w = (size_t)g.Co * taps * g.Ci;
  const int sp = COT == 128 ? split_id : 2 * split_id + wh;
  float* out = part + (size_t)sp * (n_w + g.Co);
  const int ci = ci0 + 32 * wc + (l & 31);
  const int cob = co0 + 32 * cb0;
#pragma unroll
  for (int n = 0; n < NT; ++n) {
    const int ta = ta0 + n / KW, tb = n % KW;
    if (ta >= g.kh || ci >= g.Ci) continue;
    const int tap = ta * g.kw + tb;
#pragma unroll
    for (int i = 0; i < AI; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int co = cob + 32 * i + 8 * (r >> 2) + 4 * (l >> 5) + (r & 3);
        if (co < g.Co) out[((size_t)co * taps + tap) * g.Ci + ci] = acc[i][n][r];
      }
  }
  if (do_bias && (l & 31) == 0) {  // every column of accb holds the row sums of dz
#pragma unroll
    for (int i = 0; i < AI; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int co = cob + 32 * i + 8 * (r >> 2) + 4 * (l >> 5) + (r & 3);
        if (co < g.Co) out[n_w + co] = accb[i][r];
      }
  }
}

struct TrPlan {
  int gr, kw, cot, tap_groups, tiles, splits, chunks_per_split, partials;
};

// filter rows per workgroup: all taps of a group are accumulated together, at most 9 accumulator pairs
int rows_per_group(int kh, int kw) {
  if (kw == 1) return kh >= 3 ? 3 : 1;
  if (kw == 3) return kh >= 3 ? 3 : 1;
  return 1;  // kw = 5, 7: one filter row per workgroup
}

bool make_plan(const ConvGeom& g, TrPlan& p) {
  // stride 1 with at most "same" padding: Ho <= H, Wo <= W (the kernel numbers pixels by INPUT rows and columns and
  // reads dz as zero where a position has no output)
  if (g.stride != 1 || g.up > 1) return false;
  if (g.ph < 0 || g.pw < 0 || 2 * g.ph > g.kh - 1 || 2 * g.pw > g.kw - 1) return false;
  if (g.Ho != g.H + 2 * g.ph - g.kh + 1 || g.Wo != g.W + 2 * g.pw - g.kw + 1 || g.Ho < 1 || g.Wo < 1) return false;
  if (g.kw != 1 && g.kw != 3 && g.kw != 5 && g.kw != 7) return false;
  if ((g.Ci % 8) || (g.Co % 8) || g.Ci < 32) return false;
  const long long V = (long long)g.N * g.H * (g.W + g.pw);
  if (V + 2 * kPix >= (1ll << 31) || (long long)g.N * g.H * g.W * (g.Ci > g.Co ? g.Ci : g.Co) >= (1ll << 40)) return false;
  p.kw = g.kw;
  p.gr = rows_per_group(g.kh, g.kw);
  if (p.gr == 3 && g.kh == 1) return false;
  p.tap_groups = (g.kh + p.gr - 1) / p.gr;
  p.cot = g.Co <= 64 ? 64 : 128;
  p.tiles = ((g.Co + p.cot - 1) / p.cot) * ((g.Ci + 63) / 64) * p.tap_groups;
  const int nchunks = (int)((V + kPix - 1) / kPix);
  int s = (256 + p.tiles / 2) / p.tiles;  // about one workgroup per compute unit
  if (s > nchunks / 4) s = nchunks / 4;
  if (s < 1) s = 1;
  p.chunks_per_split = (nchunks + s - 1) / s;
  p.splits = (nchunks + p.chunks_per_split - 1) / p.chunks_per_split;
  p.partials = p.cot == 64 ? 2 * p.splits : p.splits;
  return true;
}

template <int GR, int KW>
void launch_tr(hipStream_t s, const TrPlan& p, const bf16_t* dz, const bf16_t* x, float* part, const ConvGeom& g) {
  constexpr int AI = 2 * (GR * KW + 1) <= 16 ? 2 : 1;  // accumulator tiles per wave: AI * (taps + bias) <= 16
  const dim3 grid(p.tiles, p.splits);
  if (p.cot == 128)
    conv_wgrad_tr_kernel<GR, KW, 128, AI><<<grid, 512 / AI, 0, s>>>(dz, x, part, g, p.chunks_per_split, p.tap_groups);
  else
    conv_wgrad_tr_kernel<GR, KW, 64, AI><<<grid, 512 / AI, 0, s>>>(dz, x, part, g, p.chunks_per_split, p.tap_groups);
}

}  // namespace

int conv_wgrad_tr_partials(const ConvGeom& g) {
  TrPlan p;
  return make_plan(g, p) ? p.partials : 0;
}

hipError_t conv_wgrad_tr_partial_bf16(hipStream_t s, const bf16_t* dz, const bf16_t* x, float* part, int partials,
                                      const ConvGeom& g) {
  TrPlan p;
  if (!make_plan(g, p) || partials != p.partials) return hipErrorInvalidValue;
  if ((reinterpret_cast<uintptr_t>(dz) | reinterpret_cast<uintptr_t>(x)) & 15) return hipErrorInvalidValue;
  if (p.gr == 3 && p.kw == 3) launch_tr<3, 3>(s, p, dz, x, part, g);
  else if (p.gr == 3 && p.kw == 1) launch_tr<3, 1>(s, p, dz, x, part, g);
  else if (p.gr == 1 && p.kw == 1) launch_tr<1, 1>(s, p, dz, x, part, g);
  else if (p.gr == 1 && p.kw == 3) launch_tr<1, 3>(s, p, dz, x, part, g);
  else if (p.gr == 1 && p.kw == 5) launch_tr<1, 5>(s, p, dz, x, part, g);
  else if (p.gr == 1 && p.kw == 7) launch_tr<1, 7>(s, p, dz, x, part, g);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace pd
