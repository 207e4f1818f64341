// bf16 x bf16 -> fp32-accumulate GEMM kernels for gfx950 (CDNA4), built on the 32x32x16 bf16 MFMA.
//
// Three contractions of a Linear layer inside a pipeline stage:
//   forward   y  = act(x w^T + b)          reduction over in-features, both operands reduction-contiguous
//             (skinny_dma_kernel: tiles straight from global memory into LDS; gemm_kernel<false>: through
//             registers, for reductions that are not a multiple of 128)
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
#include <type_traits>

#include "bf16_util.h"
#include "mfma_util.h"
#include "pd_kernels.h"

namespace pd {
namespace {

constexpr int BM = 64;  // rows of the skinny GEMM's output tile (minibatch direction)

// ------------------------------------------------------------------------------------------------
// Skinny GEMM for forward and dgrad:  out[M][C] = A[M][R] * B, fp32 accumulate, then the epilogue.
//   BT = false (forward): B is w[C][R], reduction contiguous:   out = x w^T (+ bias, ReLU)
//   BT = true  (dgrad):   B is w[R][C], reduction rows:         out = dz w  (.* ReLU mask); every 2x8 block
//                         of w is transposed on its way into LDS
// grid = (ceil(C/BN), ceil(M/BM), splits).  Each workgroup reduces a contiguous range of BK-wide stages.
// The weight matrix is read once from HBM, so what matters is bytes in flight: global loads run PD stages
// ahead of the MFMAs in registers, LDS is double-buffered.
// With splits > 1 the partial tiles go to `ws` and splitk_epilogue_kernel finishes the job.
// ------------------------------------------------------------------------------------------------
struct GemmEpilogue {
  const bf16_t* bias;  // forward: [C] or null
  const bf16_t* mask;  // dgrad: [M][C], value kept where mask > 0; or null
  int relu;            // forward
  bf16_t* out;         // [M][C] bf16, used when out_f is null
  float* out_f;        // [M][C] fp32 (logits for the loss), or null
};

__device__ __forceinline__ void gemm_store(const GemmEpilogue& ep, float v, int m, int c, int C) {
  const size_t off = (size_t)m * C + c;
  if (ep.bias) v += bf2f(ep.bias[c]);
  if (ep.relu) v = fmaxf(v, 0.f);
  if (ep.out_f) {
    ep.out_f[off] = v;
    return;
  }
  uint16_t o = f2bf(v);
  if (ep.mask && !bf_positive(ep.mask[off])) o = 0;
  ep.out[off] = o;
}

// Tile shape: BM_ x BN_ outputs, BK_ reduction elements per stage; PD stages of global loads in flight in
// registers; NBUF LDS buffers (1: store / barrier / compute; 2: the store of the next stage overlaps compute).
// BK_ sets how many contiguous bytes of each weight row a workgroup touches per visit (2*BK_): the weight
// stream is the HBM traffic, and short per-row visits scattered over many rows waste DRAM page locality.
template <bool BT, int BN_, int BK_, int PD, int NBUF>
__global__ __launch_bounds__(kThreads) void gemm_kernel(const bf16_t* __restrict__ A, const bf16_t* __restrict__ Bm,
                                                        GemmEpilogue ep, float* __restrict__ ws, int M, int C, int R,
                                                        int splits, int lda, int partial_only) {
  constexpr int LDA = BK_ + 8;             // padded row (bf16) of a reduction-contiguous tile
  constexpr int G = BK_ / 8;               // 16-byte groups per row
  constexpr int ACH = BM * G / kThreads;   // 16-byte chunks of A per thread and stage
  constexpr int BCH = BN_ * G / kThreads;  // ... of B
  constexpr int WN = BN_ / 32;             // waves along the output columns
  constexpr int WM = 4 / WN;               // waves along the rows
  constexpr int MB = (BM / 32) / WM;       // 32-row blocks per wave
  constexpr int kAElems = BM * LDA;
  constexpr int kBWords = BN_ * LDA / 2;   // covers both B layouts (plain: BN_*LDA bf16; transposed: BN_*BK_/2 words)
  static_assert(ACH >= 1 && BCH >= 2 && (BCH % 2) == 0 && MB >= 1, "tile shape");
  __shared__ __attribute__((aligned(16))) bf16_t As[NBUF][kAElems];
  __shared__ __attribute__((aligned(16))) uint32_t Bs[NBUF][kBWords];
  const int t = threadIdx.x, l = t & 63, w = t >> 6;
  const int wn = w % WN, wm = w / WN;
  const int c0 = blockIdx.x * BN_, m0 = blockIdx.y * BM, z = blockIdx.z;
  const int T = (R + BK_ - 1) / BK_;
  const int rt0 = (int)((long long)z * T / splits), rt1 = (int)((long long)(z + 1) * T / splits);

  struct Regs {
    uint4 a[ACH], b[BCH];
  };
  // with a single row tile every weight is read exactly once by the whole grid: stream it past the caches
  const bool once = gridDim.y == 1;
  auto ldw = [&](const bf16_t* p) { return once ? ldg16_stream(p) : ldg16(p); };
  auto gload = [&](Regs& r, int rt) {
    const int r0 = rt * BK_;
    const bool live = rt < rt1;
#pragma unroll
    for (int i = 0; i < ACH; ++i) {
      const int c = t + kThreads * i, row = c / G, rr = r0 + (c % G) * 8, m = m0 + row;
      r.a[i] = (live && m < M && rr < R) ? ldg16(A + (size_t)m * lda + rr) : zero16();
    }
    if (!BT) {
#pragma unroll
      for (int i = 0; i < BCH; ++i) {
        const int c = t + kThreads * i, row = c / G, rr = r0 + (c % G) * 8, cc = c0 + row;
        r.b[i] = (live && cc < C && rr < R) ? ldw(Bm + (size_t)cc * R + rr) : zero16();
      }
    } else {
#pragma unroll
      for (int i = 0; i < BCH / 2; ++i) {
        const int b = t + kThreads * i, cch = b % (BN_ / 8), pair = b / (BN_ / 8);
        const int rr = r0 + 2 * pair, cc = c0 + 8 * cch;
        r.b[2 * i] = (live && rr < R && cc < C) ? ldw(Bm + (size_t)rr * C + cc) : zero16();
        r.b[2 * i + 1] = (live && rr + 1 < R && cc < C) ? ldw(Bm + (size_t)(rr + 1) * C + cc) : zero16();
      }
    }
  };
  auto sstore = [&](int buf, const Regs& r) {
#pragma unroll
    for (int i = 0; i < ACH; ++i) {
      const int c = t + kThreads * i;
      *reinterpret_cast<uint4*>(&As[buf][(c / G) * LDA + (c % G) * 8]) = r.a[i];
    }
    if (!BT) {
      bf16_t* bs = reinterpret_cast<bf16_t*>(Bs[buf]);
#pragma unroll
      for (int i = 0; i < BCH; ++i) {
        const int c = t + kThreads * i;
        *reinterpret_cast<uint4*>(&bs[(c / G) * LDA + (c % G) * 8]) = r.b[i];
      }
    } else {
#pragma unroll
      for (int i = 0; i < BCH / 2; ++i) {
        const int b = t + kThreads * i, cch = b % (BN_ / 8), pair = b / (BN_ / 8);
        store_transposed_pair<G>(Bs[buf], 8 * cch, pair, r.b[2 * i], r.b[2 * i + 1]);
      }
    }
  };
  f32x16 acc[MB];
#pragma unroll
  for (int i = 0; i < MB; ++i) acc[i] = f32x16{0};
  auto compute = [&](int buf) {
    const bf16_t* bs = reinterpret_cast<const bf16_t*>(Bs[buf]);
    const int brow = 32 * wn + (l & 31);
#pragma unroll
    for (int ks = 0; ks < BK_ / 16; ++ks) {
      const int kk = ks * 16 + (l >> 5) * 8;
      const uint4 b = BT ? load_swizzled_frag<G>(Bs[buf], brow, 2 * ks + (l >> 5))
                         : *reinterpret_cast<const uint4*>(&bs[brow * LDA + kk]);
#pragma unroll
      for (int i = 0; i < MB; ++i) {
        const uint4 a = *reinterpret_cast<const uint4*>(&As[buf][(32 * (MB * wm + i) + (l & 31)) * LDA + kk]);
        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(a), frag(b), acc[i], 0, 0, 0);
      }
    }
  };

  if (rt0 < rt1) {
    Regs Rg[PD];
#pragma unroll
    for (int p = 0; p < PD; ++p) gload(Rg[p], rt0 + p);
    if (NBUF == 2) {
      sstore(0, Rg[0]);
      gload(Rg[0], rt0 + PD);
      __syncthreads();
    }
    for (int base = rt0; base < rt1; base += PD) {
#pragma unroll
      for (int j = 0; j < PD; ++j) {
        const int rt = base + j;
        if (rt >= rt1) break;
        if (NBUF == 2) {
          const int cur = (rt - rt0) & 1;
          compute(cur);
          if (rt + 1 < rt1) {  // stage rt+1 sits in register slot (j+1) % PD; refill that slot PD stages ahead
            sstore(cur ^ 1, Rg[(j + 1) % PD]);
            gload(Rg[(j + 1) % PD], rt + 1 + PD);
          }
          __syncthreads();
        } else {
          sstore(0, Rg[j]);             // stage rt sits in register slot j
          gload(Rg[j], rt + PD);
          __syncthreads();
          compute(0);
          __syncthreads();
        }
      }
    }
  }

  const int c = c0 + 32 * wn + (l & 31);
  if (c >= C) return;
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int m = m0 + 32 * (MB * wm + i) + 8 * (r >> 2) + 4 * (l >> 5) + (r & 3);
      if (m >= M) continue;
      if (splits == 1 && !partial_only) gemm_store(ep, acc[i][r], m, c, C);
      else ws[((size_t)z * M + m) * C + c] = acc[i][r];
    }
}

// Sums the split-K partial tiles in split order (a fixed order: deterministic) and applies the epilogue.
// One thread per 4 consecutive columns of one row (C is a multiple of 4).  Runs as its own launch: on this
// multi-die part a device-scope release/acquire inside the GEMM (to let the last workgroup of a tile reduce) costs
// an L2 write-back per workgroup, far more than a second small kernel.  Every load is issued before the first value
// is needed: the partial tiles in batches of eight (unconditional loads of a clamped split index; a surplus load
// is dropped by a select, not by a branch), bias and mask as one 8-byte load each next to the first batch; the
// result leaves as one 8- or 16-byte store.  (At 64 x 4096 outputs the launch takes 4.7 us either way, which is
// what any launch that depends on its predecessor takes on this chip; the batching matters for many splits.)
__global__ __launch_bounds__(256) void splitk_epilogue_kernel(const float* __restrict__ ws, int splits, int M, int C,
                                                              GemmEpilogue ep) {
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t total4 = (size_t)M * C / 4;
  if (idx >= total4) return;
  const size_t e = idx * 4, plane = (size_t)M * C;
  const int m = (int)(e / C), c = (int)(e % C);
  constexpr int kBatch = 8;
  const bool vec = ((reinterpret_cast<uintptr_t>(ep.bias) | reinterpret_cast<uintptr_t>(ep.mask) |
                     reinterpret_cast<uintptr_t>(ep.out)) & 7) == 0 &&
                   (reinterpret_cast<uintptr_t>(ep.out_f) & 15) == 0;
  uint2 bias4 = make_uint2(0u, 0u), mask4 = make_uint2(0x3f803f80u, 0x3f803f80u);  // no mask: every element kept
  if (vec) {
    if (ep.bias) bias4 = *reinterpret_cast<const uint2*>(ep.bias + c);
    if (ep.mask && !ep.out_f) mask4 = *reinterpret_cast<const uint2*>(ep.mask + e);
  }
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int z0 = 0; z0 < splits; z0 += kBatch) {
    float4 p[kBatch];
#pragma unroll
    for (int q = 0; q < kBatch; ++q) {
      const int z = z0 + q < splits ? z0 + q : splits - 1;
      p[q] = *reinterpret_cast<const float4*>(ws + (size_t)z * plane + e);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int q = 0; q < kBatch; ++q) {
      const bool live = z0 + q < splits;
      if (z0 + q == 0) {
        s = p[q];  // the first tile starts the sum (not 0 + tile: keeps the sign of a zero)
      } else {
        s.x = live ? s.x + p[q].x : s.x; s.y = live ? s.y + p[q].y : s.y;
        s.z = live ? s.z + p[q].z : s.z; s.w = live ? s.w + p[q].w : s.w;
      }
    }
  }
  if (!vec) {
    gemm_store(ep, s.x, m, c, C);
    gemm_store(ep, s.y, m, c + 1, C);
    gemm_store(ep, s.z, m, c + 2, C);
    gemm_store(ep, s.w, m, c + 3, C);
    return;
  }
  float v[4] = {s.x, s.y, s.z, s.w};
  const uint16_t bb[4] = {(uint16_t)(bias4.x & 0xffffu), (uint16_t)(bias4.x >> 16), (uint16_t)(bias4.y & 0xffffu),
                          (uint16_t)(bias4.y >> 16)};
  const uint16_t mk[4] = {(uint16_t)(mask4.x & 0xffffu), (uint16_t)(mask4.x >> 16), (uint16_t)(mask4.y & 0xffffu),
                          (uint16_t)(mask4.y >> 16)};
  uint16_t o[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    if (ep.bias) v[k] += bf2f(bb[k]);
    if (ep.relu) v[k] = fmaxf(v[k], 0.f);
    o[k] = f2bf(v[k]);
    if (!bf_positive(mk[k])) o[k] = 0;
  }
  if (ep.out_f) {
    *reinterpret_cast<float4*>(ep.out_f + e) = make_float4(v[0], v[1], v[2], v[3]);
  } else {
    uint2 pk;
    pk.x = (uint32_t)o[0] | ((uint32_t)o[1] << 16);
    pk.y = (uint32_t)o[2] | ((uint32_t)o[3] << 16);
    *reinterpret_cast<uint2*>(ep.out + e) = pk;
  }
}

// ------------------------------------------------------------------------------------------------
// Forward product of a minibatch-sized layer with both tiles going straight from global memory into LDS.
//   ws[z][m][c] = sum over the z-th slice of the reduction of A[m][r] * W[c][r]       (fp32 partial sums)
// 64 x BN output tile, 128 reduction elements per stage, NS stages in LDS with the loads NS - 1 stages ahead of the
// MFMAs.  A tile row is 256 bytes = 16 slots of 16 bytes; a wave-wide load fills 4 consecutive rows (lane L lands
// at 16 L) and slot s of row r holds reduction group s ^ (r & 15), applied on the global side, so that the 16-byte
// fragment reads of 16 consecutive rows cover all banks.  The four waves split the eight 16-wide reduction steps
// of a stage between them (each fragment is read from LDS once, not once per wave sharing a row or column block)
// and every wave accumulates the whole 64 x BN tile; the four partial tiles are added through LDS at the end, in
// wave order.  The loads are unconditional (rows past the matrix are clamped to its last row and feed outputs that
// are never stored; stages past the slice re-read its last stage into a buffer that is never read), so the number
// of loads in flight is fixed and the waits are explicit counts.
// Requires R % 128 == 0, 16-byte aligned rows, operands below 4 GiB (32-bit byte offsets).
// ------------------------------------------------------------------------------------------------
template <int BN, int NS>
__global__ __launch_bounds__(kThreads) void skinny_dma_kernel(const bf16_t* __restrict__ A, int lda,
                                                              const bf16_t* __restrict__ W, float* __restrict__ ws,
                                                              int M, int C, int R, int splits) {
  constexpr int SK = 128, ROWB = SK * 2, ATILE = BM * ROWB, STAGE = (BM + BN) * ROWB;
  constexpr int QA = BM / 16, QB = BN / 16, LPS = QA + QB;  // wave-wide loads per wave and stage (4 rows each)
  constexpr int NI = BM / 32, NJ = BN / 32;
  constexpr int RED = 4 * BM * BN * 4, SMEM = NS * STAGE > RED ? NS * STAGE : RED;  // stages, then the four partial tiles
  static_assert(NS >= 2 && SMEM <= 160 * 1024, "LDS budget");
  __shared__ __attribute__((aligned(1024))) char smem[SMEM];
  const int t = threadIdx.x, l = t & 63;
  const int w = __builtin_amdgcn_readfirstlane(t >> 6);
  const int c0 = blockIdx.x * BN, m0 = blockIdx.y * BM, z = blockIdx.z;
  const int T = R / SK;
  const int rt0 = (int)((long long)z * T / splits), rt1 = (int)((long long)(z + 1) * T / splits), n = rt1 - rt0;

  uint32_t off[LPS];
#pragma unroll
  for (int q = 0; q < LPS; ++q) {
    const int row = ((q < QA ? q : q - QA) * 4 + w) * 4 + (l >> 4), g = (l & 15) ^ (row & 15);
    if (q < QA) {
      const int ra = m0 + row < M ? m0 + row : M - 1;
      off[q] = ((uint32_t)ra * (uint32_t)lda + g * 8) * 2u;
    } else {
      const int rb = c0 + row < C ? c0 + row : C - 1;
      off[q] = ((uint32_t)rb * (uint32_t)R + g * 8) * 2u;
    }
  }
  auto load_stage = [&](int buf, int sc) {  // sc: stage of this slice, clamped by the caller
    const size_t k0 = (size_t)(rt0 + sc) * SK;
    char* st = smem + buf * STAGE;
#pragma unroll
    for (int q = 0; q < LPS; ++q) {
      char* dst = st + (q < QA ? 0 : ATILE) + ((q < QA ? q : q - QA) * 4 + w) * 1024;
      if (q < QA) dma_load16(A + k0, off[q], dst);
      else if (gridDim.y == 1) dma_load16_stream(W + k0, off[q], dst);  // every weight is read once by the whole grid
      else dma_load16(W + k0, off[q], dst);
    }
  };
  // this wave's reduction steps are 2w and 2w + 1: groups 4w + (l >> 5) and, two slots on, the same with bit 1 set
  int fa[NI], fb[NJ];
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const int row = 32 * i + (l & 31);
    fa[i] = row * ROWB + (((4 * w + (l >> 5)) ^ (row & 15)) << 4);
  }
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int row = 32 * j + (l & 31);
    fb[j] = ATILE + row * ROWB + (((4 * w + (l >> 5)) ^ (row & 15)) << 4);
  }
  f32x16 acc[NI][NJ];
#pragma unroll
  for (int i = 0; i < NI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j) acc[i][j] = f32x16{0};

  if (n > 0) {
#pragma unroll
    for (int d = 0; d < NS - 1; ++d) load_stage(d, d < n ? d : n - 1);
    int cur = 0, fill = NS - 1;
    for (int st = 0; st < n; ++st) {
      // this wave's loads of stage st have landed (NS - 2 later stages may be in flight); after the barrier every
      // wave's have, and every wave is done reading the buffer that is filled next
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NS - 2) * LPS) : "memory");
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
      load_stage(fill, st + NS - 1 < n ? st + NS - 1 : n - 1);
      const char* sc = smem + cur * STAGE;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        uint4 a[NI], b[NJ];
#pragma unroll
        for (int i = 0; i < NI; ++i) a[i] = *reinterpret_cast<const uint4*>(sc + (fa[i] ^ (h << 5)));
#pragma unroll
        for (int j = 0; j < NJ; ++j) b[j] = *reinterpret_cast<const uint4*>(sc + (fb[j] ^ (h << 5)));
#pragma unroll
        for (int i = 0; i < NI; ++i)
#pragma unroll
          for (int j = 0; j < NJ; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(a[i]), frag(b[j]), acc[i][j], 0, 0, 0);
      }
      cur = cur + 1 == NS ? 0 : cur + 1;
      fill = fill + 1 == NS ? 0 : fill + 1;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the trailing re-reads still write LDS
  }
  __syncthreads();
  float* red = reinterpret_cast<float*>(smem);  // [wave][row][column]
#pragma unroll
  for (int i = 0; i < NI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = 32 * i + 8 * (r >> 2) + 4 * (l >> 5) + (r & 3);
        red[((size_t)w * BM + row) * BN + 32 * j + (l & 31)] = acc[i][j][r];
      }
  __syncthreads();
  for (int idx = t; idx < BM * BN / 4; idx += kThreads) {
    const int row = idx / (BN / 4), c4 = (idx % (BN / 4)) * 4;
    float4 s = *reinterpret_cast<const float4*>(&red[(size_t)row * BN + c4]);
#pragma unroll
    for (int k = 1; k < 4; ++k) {
      const float4 p = *reinterpret_cast<const float4*>(&red[((size_t)k * BM + row) * BN + c4]);
      s.x += p.x; s.y += p.y; s.z += p.z; s.w += p.w;
    }
    const int m = m0 + row, c = c0 + c4;
    if (m >= M || c >= C) continue;
    float* o = ws + ((size_t)z * M + m) * C + c;
    if (c + 3 < C && (C & 3) == 0) {
      *reinterpret_cast<float4*>(o) = s;
    } else {
      const float v[4] = {s.x, s.y, s.z, s.w};
      for (int k = 0; k < 4 && c + k < C; ++k) o[k] = v[k];
    }
  }
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
constexpr int MC = 64;  // minibatch rows per reduction chunk

typedef float vf4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 nt_load4(const float* p) {
  const vf4_t v = __builtin_nontemporal_load(reinterpret_cast<const vf4_t*>(p));
  return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void nt_store4(float* p, float4 v) {
  const vf4_t t = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(t, reinterpret_cast<vf4_t*>(p));
}

// KIND: the update rule (UpdateRule::kind) as a compile-time constant.
// SPLIT: the fp32 master weights are the previous ring copy plus 16-bit remainders (WgradLayer::ring_in, rem_w)
// instead of an fp32 array: 2 + 2 bytes read and 2 more written per parameter instead of 4 and 4.
typedef unsigned int vu2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint2 nt_load_u2(const void* p) {
  const vu2_t v = __builtin_nontemporal_load(reinterpret_cast<const vu2_t*>(p));
  return make_uint2(v.x, v.y);
}
__device__ __forceinline__ void nt_store_u2(void* p, uint2 v) {
  const vu2_t t = {v.x, v.y};
  __builtin_nontemporal_store(t, reinterpret_cast<vu2_t*>(p));
}

template <int TN, int TK, bool NFAST, bool PREFETCH, int KIND, bool SPLIT>
__global__ __launch_bounds__(kThreads) void wgrad_update_kernel(WgradBatch batch) {
  // which layer this workgroup belongs to (all layers of a stage are updated by one launch)
  int li = 0;
  while (li + 1 < batch.count && blockIdx.x >= batch.layer[li].tile_end) ++li;
  const WgradLayer& L = batch.layer[li];
  const unsigned tile_id = blockIdx.x - (li ? batch.layer[li - 1].tile_end : 0u);
  const bf16_t* __restrict__ dZ = L.dz;
  const bf16_t* __restrict__ X = L.x;
  float* __restrict__ master = L.master_w;
  float* __restrict__ mom = L.mom_w;
  bf16_t* ring = L.ring_w;           // (no __restrict__: with a ring of depth 1 ring_in is the same slot; every
  const bf16_t* ring_in = L.ring_in;  // element is then read and later written by the same thread)
  uint16_t* __restrict__ rem = L.rem_w;
  float* __restrict__ master_b = L.master_b;
  float* __restrict__ mom_b = L.mom_b;
  bf16_t* __restrict__ ring_b = L.ring_b;
  const int M = L.M ? L.M : batch.M, N = L.N, K = L.K;
  const UpdateRule rule = batch.rule;
  constexpr int GLD = TK + 4;
  constexpr int kSlots = TN * TK / 4 / kThreads;  // float4 elements per thread in phase 2
  constexpr int NB = TN / 32;                     // 32-row MFMA blocks per wave (waves split the k columns)
  constexpr int KW = TK / 32;                     // 32-column blocks in the tile; waves take KW/4 each
  static_assert(TK % 128 == 0 && TN % 32 == 0, "tile shape");
  constexpr int KB = KW / 4;
  __shared__ __attribute__((aligned(16))) uint32_t smem[(TN * GLD > (TN + TK) * 32) ? TN * GLD : (TN + TK) * 32];
  uint32_t* dZt = smem;             // [TN][32 words]  rows = n, 64 minibatch rows each
  uint32_t* Xt = smem + TN * 32;    // [TK][32 words]  rows = k
  float* G = reinterpret_cast<float*>(smem);

  const int t = threadIdx.x, l = t & 63, w = t >> 6;
  const int ktiles = (K + TK - 1) / TK, ntiles = (N + TN - 1) / TN;
  const int kt = NFAST ? (int)(tile_id / ntiles) : (int)(tile_id % ktiles);
  const int nt = NFAST ? (int)(tile_id % ntiles) : (int)(tile_id / ktiles);
  const int n0 = nt * TN, k0 = kt * TK;

  // phase 0 (issued inside the first reduction chunk, AFTER that chunk's dz / x loads): master and momentum of this
  // thread's phase-2 elements.  Loads complete in issue order as far as the wait counter is concerned, so the chunk's
  // LDS stores can wait for dz / x alone only if these loads come later; and they are unconditional (an element
  // outside the matrix reads a clamped address and is ignored in phase 2), because a load that only some paths issue
  // makes the compiler wait for everything at the next use.
  static_assert(!SPLIT || PREFETCH, "the split master is only read ahead");
  float4 pw[kSlots], pm[kSlots];
  uint2 ph[kSlots], pl[kSlots];  // SPLIT: four bf16 of the previous ring copy, four remainders
  auto prefetch = [&]() {
#pragma unroll
    for (int q = 0; q < kSlots; ++q) {
      const int f = t + kThreads * q, row = f / (TK / 4), k = k0 + (f % (TK / 4)) * 4, n = n0 + row;
      const size_t off = (size_t)(n < N ? n : N - 1) * K + (k < K ? k : K - 4);
      if (SPLIT) {
        ph[q] = nt_load_u2(ring_in + off);
        pl[q] = nt_load_u2(rem + off);
      } else {
        pw[q] = nt_load4(master + off);
      }
      pm[q] = nt_load4(mom + off);
    }
  };

  // phase 1
  f32x16 acc[NB][KB];
#pragma unroll
  for (int i = 0; i < NB; ++i)
#pragma unroll
    for (int j = 0; j < KB; ++j) acc[i][j] = f32x16{0};
  auto chunk = [&](int mc, auto first) {
    {
      constexpr int ZB = TN / 8 * 32 / kThreads > 0 ? TN / 8 * 32 / kThreads : 1;  // dz blocks per thread
      constexpr int XB = TK / 8 * 32 / kThreads;                                    // x blocks per thread
      uint4 z0[ZB], z1[ZB], x0[XB], x1[XB];
#pragma unroll
      for (int i = 0; i < ZB; ++i) {
        const int b = t + kThreads * i, nc = b % (TN / 8), pair = b / (TN / 8);
        const int m = mc + 2 * pair, n = n0 + 8 * nc;
        const bool in = pair < 32;
        z0[i] = (in && m < M && n < N) ? ldg16(dZ + (size_t)m * N + n) : zero16();
        z1[i] = (in && m + 1 < M && n < N) ? ldg16(dZ + (size_t)(m + 1) * N + n) : zero16();
      }
#pragma unroll
      for (int i = 0; i < XB; ++i) {
        const int b = t + kThreads * i, kc = b % (TK / 8), p2 = b / (TK / 8);
        const int mm = mc + 2 * p2, k = k0 + 8 * kc;
        x0[i] = (mm < M && k < K) ? ldg16(X + (size_t)mm * K + k) : zero16();
        x1[i] = (mm + 1 < M && k < K) ? ldg16(X + (size_t)(mm + 1) * K + k) : zero16();
      }
      if (decltype(first)::value) {
        if (PREFETCH) prefetch();
      } else {
        __syncthreads();  // previous chunk's fragments fully read
      }
#pragma unroll
      for (int i = 0; i < ZB; ++i) {
        const int b = t + kThreads * i, nc = b % (TN / 8), pair = b / (TN / 8);
        if (pair < 32) store_transposed_pair<8>(dZt, 8 * nc, pair, z0[i], z1[i]);
      }
#pragma unroll
      for (int i = 0; i < XB; ++i) {
        const int b = t + kThreads * i, kc = b % (TK / 8), p2 = b / (TK / 8);
        store_transposed_pair<8>(Xt, 8 * kc, p2, x0[i], x1[i]);
      }
    }
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < MC / 16; ++ks) {
      const int g = 2 * ks + (l >> 5);
      uint4 a[NB];
#pragma unroll
      for (int i = 0; i < NB; ++i) a[i] = load_swizzled_frag<8>(dZt, 32 * i + (l & 31), g);
#pragma unroll
      for (int j = 0; j < KB; ++j) {
        const uint4 b = load_swizzled_frag<8>(Xt, 32 * (KB * w + j) + (l & 31), g);
#pragma unroll
        for (int i = 0; i < NB; ++i)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(a[i]), frag(b), acc[i][j], 0, 0, 0);
      }
    }
  };
  chunk(0, std::true_type{});
  for (int mc = MC; mc < M; mc += MC) chunk(mc, std::false_type{});
  __syncthreads();  // all fragment reads done before the tile memory is reused

  // phase 2a: accumulators -> LDS, G[n][k]
#pragma unroll
  for (int j = 0; j < KB; ++j) {
    const int kcol = 32 * (KB * w + j) + (l & 31);
#pragma unroll
    for (int i = 0; i < NB; ++i) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int nrow = 32 * i + 8 * (r >> 2) + 4 * (l >> 5) + (r & 3);
        G[nrow * GLD + kcol] = acc[i][j][r];
      }
    }
  }
  __syncthreads();

  // phase 2b: the update, row-major
#pragma unroll
  for (int q = 0; q < kSlots; ++q) {
    const int f = t + kThreads * q, row = f / (TK / 4), c4 = (f % (TK / 4)) * 4, k = k0 + c4, n = n0 + row;
    if (n < N && k < K) {
      const size_t off = (size_t)n * K + k;
      const float4 g = *reinterpret_cast<const float4*>(&G[row * GLD + c4]);
      float4 m, wv;
      if (SPLIT) {
        m = pm[q];
        wv.x = master_merge1((uint16_t)(ph[q].x & 0xffffu), (uint16_t)(pl[q].x & 0xffffu));
        wv.y = master_merge1((uint16_t)(ph[q].x >> 16), (uint16_t)(pl[q].x >> 16));
        wv.z = master_merge1((uint16_t)(ph[q].y & 0xffffu), (uint16_t)(pl[q].y & 0xffffu));
        wv.w = master_merge1((uint16_t)(ph[q].y >> 16), (uint16_t)(pl[q].y >> 16));
      } else if (PREFETCH) {
        m = pm[q];
        wv = pw[q];
      } else {
        m = *reinterpret_cast<const float4*>(mom + off);
        wv = *reinterpret_cast<const float4*>(master + off);
      }
      if (KIND == kRuleGradOnly) {  // replicated stage: the sum over replicas comes first
        *reinterpret_cast<float4*>(master + off) = g;
        continue;
      }
      apply_update_as<KIND>(rule, g.x, m.x, wv.x); apply_update_as<KIND>(rule, g.y, m.y, wv.y);
      apply_update_as<KIND>(rule, g.z, m.z, wv.z); apply_update_as<KIND>(rule, g.w, m.w, wv.w);
      nt_store4(mom + off, m);     // streamed once per step: keep these lines out of the caches
      uint2 pk;
      if (SPLIT) {
        uint16_t r[4], lo[4];
        master_split1(wv.x, r[0], lo[0]); master_split1(wv.y, r[1], lo[1]);
        master_split1(wv.z, r[2], lo[2]); master_split1(wv.w, r[3], lo[3]);
        pk.x = (uint32_t)r[0] | ((uint32_t)r[1] << 16);
        pk.y = (uint32_t)r[2] | ((uint32_t)r[3] << 16);
        nt_store_u2(rem + off, make_uint2((uint32_t)lo[0] | ((uint32_t)lo[1] << 16), (uint32_t)lo[2] | ((uint32_t)lo[3] << 16)));
      } else {
        nt_store4(master + off, wv);
        pk.x = (uint32_t)f2bf(wv.x) | ((uint32_t)f2bf(wv.y) << 16);
        pk.y = (uint32_t)f2bf(wv.z) | ((uint32_t)f2bf(wv.w) << 16);
      }
      *reinterpret_cast<uint2*>(ring + off) = pk;  // read back by the next forward pass: ordinary store (measured:
                                                    // a non-temporal store here costs the update more than the forward gains)
    }
  }

  // bias: column sums of dz in row order, by the workgroups of the first k-tile
  if (kt == 0 && master_b && t < TN) {
    const int n = n0 + t;
    if (n < N) {
      float g = 0.f;
      for (int m = 0; m < M; ++m) g += bf2f(dZ[(size_t)m * N + n]);
      if (KIND == kRuleGradOnly) {
        master_b[n] = g;
        return;
      }
      float mv = mom_b[n], bv = master_b[n];
      apply_update_as<KIND>(rule, g, mv, bv);
      mom_b[n] = mv;
      master_b[n] = bv;
      ring_b[n] = f2bf(bv);
    }
  }
}

template <int TN, int TK, bool NFAST, bool PREFETCH>
hipError_t launch_wgrad_update(hipStream_t s, WgradBatch batch) {
  unsigned tiles = 0;
  for (int i = 0; i < batch.count; ++i) {
    tiles += (unsigned)(((batch.layer[i].K + TK - 1) / TK) * ((batch.layer[i].N + TN - 1) / TN));
    batch.layer[i].tile_end = tiles;
  }
  if (tiles == 0) return hipSuccess;
  int n_split = 0;
  for (int i = 0; i < batch.count; ++i) {
    if ((batch.layer[i].ring_in != nullptr) != (batch.layer[i].rem_w != nullptr)) return hipErrorInvalidValue;
    n_split += batch.layer[i].rem_w != nullptr;
  }
  if (n_split != 0 && n_split != batch.count) return hipErrorInvalidValue;
  if (n_split) {
    switch (batch.rule.kind) {
      case 0: wgrad_update_kernel<TN, TK, NFAST, true, 0, true><<<tiles, kThreads, 0, s>>>(batch); break;
      case 1: wgrad_update_kernel<TN, TK, NFAST, true, 1, true><<<tiles, kThreads, 0, s>>>(batch); break;
      default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
  }
  switch (batch.rule.kind) {
    case 0: wgrad_update_kernel<TN, TK, NFAST, PREFETCH, 0, false><<<tiles, kThreads, 0, s>>>(batch); break;
    case 1: wgrad_update_kernel<TN, TK, NFAST, PREFETCH, 1, false><<<tiles, kThreads, 0, s>>>(batch); break;
    case kRuleGradOnly: wgrad_update_kernel<TN, TK, NFAST, false, kRuleGradOnly, false><<<tiles, kThreads, 0, s>>>(batch); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

// Launch shapes of the register-staged kernel, picked from sweeps at the VGG16 classifier's sizes on MI355X
// (minibatch 64).  Forward (shapes the direct-to-LDS kernel does not take): 64-column tiles, 128 reduction
// elements per stage, two stages of loads in flight, two LDS buffers.  Dgrad of a large matrix: 128 x 128 tiles
// (fewer, longer transposing stages); of a small one: 64 x 256.
constexpr int kFwdBN = 64, kFwdBK = 128, kFwdPD = 2, kFwdNBUF = 2;
constexpr int kBigBN = 128, kBigBK = 128, kBigPD = 2, kBigNBUF = 1;
constexpr int kSmallBN = 64, kSmallBK = 256, kSmallPD = 1, kSmallNBUF = 1;
constexpr size_t kBigDgradElems = (size_t)32 << 20;  // weight elements from which the big dgrad shape is used
// The 256 x 256-tile kernel (gemm_big_bf16.hip) takes over once its grid fills at least half the chip's 256 CUs.
// Timed alone the large tiles already win from 48-64 tiles on (at 80 tiles, 5120 x 4000 x 1000: forward 90 vs
// 109 us, input gradient 106 vs 129 us), but with that threshold the two-stream LSTM pipeline, where such products
// run next to the other stage's kernels, got slower (5.26 vs 5.02 ms per minibatch): a workgroup that holds 128 KB
// of LDS leaves no room on its compute unit for the other stream.
constexpr int kDefaultBigMinTiles = 128;
int g_big_min_tiles = kDefaultBigMinTiles;
bool use_big_tiles(int rows, int cols) { return ((rows + 255) / 256) * ((cols + 255) / 256) >= g_big_min_tiles; }

// Enough workgroups to fill the chip (about two per CU, all co-resident), never more splits than stages.
int pick_splits(int tiles, int red_tiles) {
  int s = 512 / tiles;
  if (s > red_tiles / 2) s = red_tiles / 2;
  if (s > 32) s = 32;
  if (s < 1) s = 1;
  return s;
}

template <int BN_, int BK_>
size_t splitk_bytes_t(int rows, int cols, int red) {
  const int tiles = ((cols + BN_ - 1) / BN_) * ((rows + BM - 1) / BM);
  const int s = pick_splits(tiles, (red + BK_ - 1) / BK_);
  return s > 1 ? (size_t)s * rows * cols * sizeof(float) : (size_t)0;
}

// lda = row stride of A (0: dense, = R).  splits_out != null: leave the fp32 partial sums ws[split][M][C]
// (at least one) for the caller's own epilogue and report how many there are.
// The direct-to-LDS forward kernel, when the shape allows it (see the kernel) and the workspace holds its partial
// sums.  Returns false if the register-staged kernel has to do the job.  Measured at 64 x 4096 x 25088 on MI355X,
// epilogue launch (4.7 us) included, with cached weight loads, which repeated calls partly serve from the 256 MB
// memory-side cache: 64 columns and 3 stages on 256 workgroups 39.6 us, 4 stages 40.1, 2 stages on 512 workgroups
// 41.9, 128 columns and 3 stages 42.9.  With the non-temporal weight loads the kernel uses (cached ones made the
// update kernel later in the step 6 % slower) the chosen shape takes 46.0 us against 49.1 for the register-staged
// kernel; a kernel that only streams the weights takes 32.6, one that also fetches the activation tiles 41.2.
constexpr int kDmaBN = 64, kDmaNS = 3, kDmaWgs = 256;
template <int BN, int NS>
bool launch_skinny_dma(hipStream_t s, const bf16_t* a, const bf16_t* w, const GemmEpilogue& ep, int M, int C, int R,
                       float* ws, size_t ws_bytes, int lda, int* splits_out, int target_wgs) {
  constexpr int SK = 128;
  if (R % SK != 0 || lda % 8 != 0 || !ws) return false;
  if ((size_t)M * lda * 2 >= ((size_t)1 << 32) || (size_t)C * R * 2 >= ((size_t)1 << 32)) return false;
  if ((reinterpret_cast<uintptr_t>(a) | reinterpret_cast<uintptr_t>(w)) & 15) return false;
  const int tc = (C + BN - 1) / BN, tm = (M + BM - 1) / BM, T = R / SK;
  int splits = target_wgs / (tc * tm);
  if (splits > T / 2) splits = T / 2;
  if (splits > 32) splits = 32;
  const size_t fit = ws_bytes / ((size_t)M * C * sizeof(float));
  if ((size_t)splits > fit) splits = (int)fit;
  if (splits < 2) return false;
  skinny_dma_kernel<BN, NS><<<dim3(tc, tm, splits), kThreads, 0, s>>>(a, lda, w, ws, M, C, R, splits);
  if (splits_out) {
    *splits_out = splits;
    return true;
  }
  const size_t total4 = (size_t)M * C / 4;
  splitk_epilogue_kernel<<<(unsigned)((total4 + 255) / 256), 256, 0, s>>>(ws, splits, M, C, ep);
  return true;
}

template <bool BT, int BN_, int BK_, int PD, int NBUF>
hipError_t launch_gemm(hipStream_t s, const bf16_t* a, const bf16_t* b, const GemmEpilogue& ep, int M, int C, int R,
                       float* ws, size_t ws_bytes, int lda = 0, int* splits_out = nullptr) {
  if (!BT && launch_skinny_dma<kDmaBN, kDmaNS>(s, a, b, ep, M, C, R, ws, ws_bytes, lda ? lda : R, splits_out, kDmaWgs))
    return hipGetLastError();
  const int tc = (C + BN_ - 1) / BN_, tm = (M + BM - 1) / BM;
  int splits = pick_splits(tc * tm, (R + BK_ - 1) / BK_);
  if (splits > 1 && (!ws || (size_t)splits * M * C * sizeof(float) > ws_bytes)) splits = 1;
  dim3 grid(tc, tm, splits);
  if (splits_out) {
    if (!ws || (size_t)M * C * sizeof(float) > ws_bytes) return hipErrorInvalidValue;
    *splits_out = splits;
    gemm_kernel<BT, BN_, BK_, PD, NBUF><<<grid, kThreads, 0, s>>>(a, b, ep, ws, M, C, R, splits, lda ? lda : R, 1);
    return hipGetLastError();
  }
  gemm_kernel<BT, BN_, BK_, PD, NBUF><<<grid, kThreads, 0, s>>>(a, b, ep, ws, M, C, R, splits, lda ? lda : R, 0);
  if (splits > 1) {
    const size_t total4 = (size_t)M * C / 4;
    splitk_epilogue_kernel<<<(unsigned)((total4 + 255) / 256), 256, 0, s>>>(ws, splits, M, C, ep);
  }
  return hipGetLastError();
}

}  // namespace

int set_big_tile_threshold(int min_tiles) {
  const int old = g_big_min_tiles;
  if (min_tiles >= 1) g_big_min_tiles = min_tiles;
  return old;
}

// How a product with `rows` x `cols` outputs and reduction length `red` runs on the 256 x 256-tile kernels:
//   1   the output tiles alone fill the chip;
//   > 1 too few tiles for that, but many rows and a long reduction: the reduction is split this many ways over about
//       one workgroup per compute unit, the fp32 partial products are added up by splitk_epilogue_kernel
//       (`red_step`: the kernel's stage length, which the reduction must be a multiple of);
//   0   not a case for the large tiles (the kernels built for minibatch-sized row counts take it).
// Measured on MI355X (8192 -> 1024 rows at 4096 x 25088): the forward product of 1024 rows 459 us on the small-tile
// split-K kernel; the input gradient of 5120 rows against 30000 x 1000 weights 129 us on an idle chip.
int big_tile_splits(int rows, int cols, int red, int red_step) {
  const int tiles = ((rows + 255) / 256) * ((cols + 255) / 256);
  const int whole = tiles >= g_big_min_tiles ? 1 : 0;     // what applies if the reduction is not split
  if (g_big_min_tiles != kDefaultBigMinTiles) return whole;  // a forced threshold means exactly that
  if (rows < 256 || red < 2048 || (red % red_step) != 0 || (cols % 4) != 0) return whole;
  int s = 256 / tiles;  // (also for exactly 128 tiles, which would leave half of the compute units idle)
  if (s > red / 512) s = red / 512;
  if (s > 16) s = 16;
  return s >= 2 ? s : whole;
}

bool linear_fwd_uses_big_tiles(int M, int N) { return use_big_tiles(M, N); }

size_t gemm_bf16_workspace_bytes(int M, int N, int K) {
  const int sf = big_tile_splits(M, N, K, 64), sd = big_tile_splits(M, K, N, 8);
  const size_t a = sf == 1 ? 0 : sf > 1 ? (size_t)sf * M * N * sizeof(float) : splitk_bytes_t<kFwdBN, kFwdBK>(M, N, K);
  const size_t b = sd == 1 ? linear_dgrad_big_scratch_bytes(N, K)  // room for transposed weights
                   : sd > 1 ? (size_t)sd * M * K * sizeof(float)
                   : (size_t)N * K >= kBigDgradElems ? splitk_bytes_t<kBigBN, kBigBK>(M, K, N)
                                                     : splitk_bytes_t<kSmallBN, kSmallBK>(M, K, N);
  return a > b ? a : b;
}

hipError_t linear_fwd_bf16(hipStream_t s, const bf16_t* x, const bf16_t* w, const bf16_t* b, bf16_t* y, float* y_f32,
                           int M, int N, int K, bool relu, float* ws, size_t ws_bytes) {
  const int sp = big_tile_splits(M, N, K, 64);
  if (sp == 1) return linear_fwd_big_bf16(s, x, K, w, b, y, y_f32, M, N, K, relu, 1, nullptr);
  GemmEpilogue ep = {b, nullptr, relu ? 1 : 0, y, y_f32};
  if (sp > 1 && ws && (size_t)sp * M * N * sizeof(float) <= ws_bytes &&
      linear_fwd_big_bf16(s, x, K, w, nullptr, nullptr, nullptr, M, N, K, false, sp, ws) == hipSuccess) {
    const size_t total4 = (size_t)M * N / 4;
    splitk_epilogue_kernel<<<(unsigned)((total4 + 255) / 256), 256, 0, s>>>(ws, sp, M, N, ep);
    return hipGetLastError();
  }
  return launch_gemm<false, kFwdBN, kFwdBK, kFwdPD, kFwdNBUF>(s, x, w, ep, M, N, K, ws, ws_bytes);
}

hipError_t linear_dgrad_bf16(hipStream_t s, const bf16_t* dz, const bf16_t* w, const bf16_t* mask, bf16_t* dx, int M,
                             int N, int K, float* ws, size_t ws_bytes) {
  const int sp = big_tile_splits(M, K, N, 8);
  if (sp == 1) return linear_dgrad_big_bf16(s, dz, w, mask, dx, M, N, K, ws, ws_bytes, 1);
  if (sp > 1 && ws && (size_t)sp * M * K * sizeof(float) <= ws_bytes &&
      linear_dgrad_big_bf16(s, dz, w, nullptr, nullptr, M, N, K, ws, ws_bytes, sp) == hipSuccess) {
    GemmEpilogue epr = {nullptr, mask, 0, dx, nullptr};
    const size_t total4 = (size_t)M * K / 4;
    splitk_epilogue_kernel<<<(unsigned)((total4 + 255) / 256), 256, 0, s>>>(ws, sp, M, K, epr);
    return hipGetLastError();
  }
  GemmEpilogue ep = {nullptr, mask, 0, dx, nullptr};
  if ((size_t)N * K >= kBigDgradElems)
    return launch_gemm<true, kBigBN, kBigBK, kBigPD, kBigNBUF>(s, dz, w, ep, M, K, N, ws, ws_bytes);
  return launch_gemm<true, kSmallBN, kSmallBK, kSmallPD, kSmallNBUF>(s, dz, w, ep, M, K, N, ws, ws_bytes);
}

hipError_t gemm_partial_bf16(hipStream_t s, bool w_rows_are_reduction, const bf16_t* a, int lda, const bf16_t* w, int M,
                             int C, int R, float* ws, size_t ws_bytes, int* splits_out) {
  GemmEpilogue ep = {nullptr, nullptr, 0, nullptr, nullptr};
  if (!w_rows_are_reduction)
    return launch_gemm<false, kFwdBN, kFwdBK, kFwdPD, kFwdNBUF>(s, a, w, ep, M, C, R, ws, ws_bytes, lda, splits_out);
  return launch_gemm<true, kSmallBN, kSmallBK, kSmallPD, kSmallNBUF>(s, a, w, ep, M, C, R, ws, ws_bytes, lda, splits_out);
}

hipError_t linear_wgrad_update_bf16(hipStream_t s, const WgradBatch& batch) {
  if (batch.count < 0 || batch.count > kMaxWgradLayers) return hipErrorInvalidValue;
  return launch_wgrad_update<32, 128, false, true>(s, batch);
}

}  // namespace pd
