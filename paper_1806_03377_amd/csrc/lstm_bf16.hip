// Element-wise halves of an LSTM time step (the matrix halves are the GEMM kernels).  fp32 throughout;
// only the hidden state and the gate pre-activation gradients, which feed MFMA GEMMs, are rounded to bf16.
#include "bf16_util.h"
#include "mfma_util.h"
#include "pd_kernels.h"

#include <mutex>
#include <set>
#include <utility>

namespace pd {
namespace {

__device__ __forceinline__ float sigmoidf(float a) { return 1.f / (1.f + expf(-a)); }

__global__ __launch_bounds__(256) void lstm_cell_fwd_kernel(float* __restrict__ gates, const float* __restrict__ rec,
                                                            int splits, const float* __restrict__ c_prev,
                                                            float* __restrict__ c, bf16_t* __restrict__ h, int B,
                                                            int H) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= B * H) return;
  const int b = idx / H, j = idx - b * H;
  float a[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const size_t e = (size_t)b * 4 * H + q * H + j;
    float v = gates[e];
    for (int s = 0; s < splits; ++s) v += rec[(size_t)s * B * 4 * H + e];
    a[q] = v;
  }
  const float ig = sigmoidf(a[0]), fg = sigmoidf(a[1]), gg = tanhf(a[2]), og = sigmoidf(a[3]);
  const float cv = fg * (c_prev ? c_prev[idx] : 0.f) + ig * gg;
  const size_t e0 = (size_t)b * 4 * H + j;
  gates[e0] = ig; gates[e0 + H] = fg; gates[e0 + 2 * H] = gg; gates[e0 + 3 * H] = og;
  c[idx] = cv;
  h[idx] = f2bf(og * tanhf(cv));
}

__global__ __launch_bounds__(256) void lstm_cell_bwd_kernel(const bf16_t* __restrict__ dh_out,
                                                            const float* __restrict__ rec, int splits,
                                                            float* __restrict__ dc, const float* __restrict__ gates,
                                                            const float* __restrict__ c, const float* __restrict__ c_prev,
                                                            bf16_t* __restrict__ da, int B, int H) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= B * H) return;
  const int b = idx / H, j = idx - b * H;
  float dh = dh_out ? bf2f(dh_out[idx]) : 0.f;
  for (int s = 0; s < splits; ++s) dh += rec[(size_t)s * B * H + idx];
  const size_t e0 = (size_t)b * 4 * H + j;
  const float ig = gates[e0], fg = gates[e0 + H], gg = gates[e0 + 2 * H], og = gates[e0 + 3 * H];
  const float tc = tanhf(c[idx]);
  const float dcv = dc[idx] + dh * og * (1.f - tc * tc);
  const float cp = c_prev ? c_prev[idx] : 0.f;
  da[e0] = f2bf(dcv * gg * ig * (1.f - ig));
  da[e0 + H] = f2bf(dcv * cp * fg * (1.f - fg));
  da[e0 + 2 * H] = f2bf(dcv * ig * (1.f - gg * gg));
  da[e0 + 3 * H] = f2bf(dh * tc * og * (1.f - og));
  dc[idx] = dcv * fg;
}


// ------------------------------------------------------------------------------------------------
// One recurrent step as ONE kernel: the skinny product with the recurrent weights and the cell update.  The
// product has few rows (the minibatch) and is read-once over a weight matrix that stays in L2, so what it costs is
// launches and latency, not flops: a workgroup owns a 16 x 16 tile of the output, its waves split the reduction
// range, every lane fetches its MFMA fragments (16 bytes, reduction-contiguous in both
// operands) straight from global memory, the waves' partial tiles are added in wave order through LDS, and the
// same threads then apply the gate non-linearities.
// ------------------------------------------------------------------------------------------------
// Uses the 16 x 16 x 32 MFMA (A fragment: row l & 15, reduction elements 8 (l >> 4) .. +7 of a 32-wide step; B
// fragment: column l & 15, same elements; D: column l & 15, rows 4 (l >> 4) + r for r = 0..3) so that a
// workgroup's tile is small and the launch has several workgroups per compute unit: these products are bound by
// memory latency, not by bandwidth or flops.
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Workgroups are dealt round-robin to the 8 XCDs, each with its own L2.  The recurrent weights are re-read at every
// time step, so the tiles are renumbered such that an XCD always works on the same contiguous range of hidden
// units (all row groups of a unit group together): its share of the weights (1/8) then stays in its L2 from
// step to step instead of every XCD streaming half of the matrix through a cache it does not fit in.
__device__ __forceinline__ void xcd_tile(int n_row_groups, int& unit_group, int& row_group) {
  const int total = gridDim.x, per = total >> 3;
  int id = blockIdx.x;
  if (id < per * 8) id = (id & 7) * per + (id >> 3);
  unit_group = id / n_row_groups;
  row_group = id - unit_group * n_row_groups;
}

// acc += A[row0 + (l & 15)][k0..k1) * brow[k0..k1)^T for one wave; k0, k1 multiples of 8.
template <int STEPS>
__device__ __forceinline__ void wave_skinny_gemm16(const bf16_t* __restrict__ arow /* this lane's A row or null */,
                                                   const bf16_t* __restrict__ brow /* this lane's B row or null */,
                                                   int k0, int k1, int l, f32x4& acc) {
  // STEPS reduction steps at a time: all their fragment loads are issued before the first MFMA, so the wave pays
  // the memory latency once per batch instead of once per step
  for (int kb = k0; kb < k1; kb += 32 * STEPS) {
    uint4 a[STEPS], b[STEPS];
#pragma unroll
    for (int st = 0; st < STEPS; ++st) {
      const int k = kb + 32 * st + 8 * (l >> 4);
      const bool live = k < k1;
      a[st] = (live && arow) ? ldg16(arow + k) : zero16();
      b[st] = (live && brow) ? ldg16(brow + k) : zero16();
    }
#pragma unroll
    for (int st = 0; st < STEPS; ++st)
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(frag(a[st]), frag(b[st]), acc, 0, 0, 0);
  }
}

// Forward: a workgroup owns 4 hidden units (their 4 x 4 = 16 gate columns) for 16 minibatch rows; grid =
// ceil(H / 4) * ceil(B / 16) workgroups (see xcd_tile); 4 waves split the reduction over H.
__global__ __launch_bounds__(256) void lstm_step_fwd_kernel(float* __restrict__ gates, const bf16_t* __restrict__ h_prev,
                                                            const bf16_t* __restrict__ whh,
                                                            const float* __restrict__ c_prev, float* __restrict__ c,
                                                            bf16_t* __restrict__ h, int B, int H) {
  __shared__ float red[4][16][17];
  const int t = threadIdx.x, l = t & 63, w = t >> 6;
  int ug, rg;
  xcd_tile((B + 15) / 16, ug, rg);
  const int u0 = ug * 4, r0 = rg * 16;
  const int kq = ((H + 127) / 128) * 32;  // reduction elements per wave (multiple of 32)
  const int k0 = w * kq, k1 = (k0 + kq) < H ? (k0 + kq) : H;
  const int cl = l & 15, unit = u0 + (cl & 3);
  const bf16_t* brow = unit < H ? whh + ((size_t)(cl >> 2) * H + unit) * H : nullptr;
  const bf16_t* arow = r0 + cl < B ? h_prev + (size_t)(r0 + cl) * H : nullptr;
  // the element-wise operands of this thread's (row, unit) are requested before the product, not after it
  const int erow = t >> 2, euu = t & 3;
  const bool eok = t < 64 && r0 + erow < B && u0 + euu < H;
  float gin[4] = {0.f, 0.f, 0.f, 0.f}, cprev = 0.f;
  if (eok) {
#pragma unroll
    for (int q = 0; q < 4; ++q) gin[q] = gates[(size_t)(r0 + erow) * 4 * H + q * H + u0 + euu];
    if (c_prev) cprev = c_prev[(size_t)(r0 + erow) * H + u0 + euu];
  }
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  if (k0 < k1) wave_skinny_gemm16<8>(arow, brow, k0, k1, l, acc);
#pragma unroll
  for (int r = 0; r < 4; ++r) red[w][4 * (l >> 4) + r][cl] = acc[r];
  __syncthreads();
  if (t < 64) {
    const int row = erow, uu = euu;
    const int b = r0 + row, j = u0 + uu;
    if (eok) {
      float a[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int col = q * 4 + uu;
        a[q] = gin[q] + (((red[0][row][col] + red[1][row][col]) + red[2][row][col]) + red[3][row][col]);
      }
      const float ig = sigmoidf(a[0]), fg = sigmoidf(a[1]), gg = tanhf(a[2]), og = sigmoidf(a[3]);
      const size_t idx = (size_t)b * H + j;
      const float cv = fg * cprev + ig * gg;
      const size_t e0 = (size_t)b * 4 * H + j;
      gates[e0] = ig; gates[e0 + H] = fg; gates[e0 + 2 * H] = gg; gates[e0 + 3 * H] = og;
      c[idx] = cv;
      h[idx] = f2bf(og * tanhf(cv));
    }
  }
}

// Backward: dh = dh_out + da_next * W_hh with W_hh^T stored [H][4H]; a workgroup owns 16 hidden units for 16
// minibatch rows; grid = ceil(H / 16) * ceil(B / 16) workgroups; 8 waves split the reduction over 4H.
__global__ __launch_bounds__(512) void lstm_step_bwd_kernel(const bf16_t* __restrict__ dh_out,
                                                            const bf16_t* __restrict__ da_next,
                                                            const bf16_t* __restrict__ whh_t, float* __restrict__ dc,
                                                            const float* __restrict__ gates, const float* __restrict__ c,
                                                            const float* __restrict__ c_prev, bf16_t* __restrict__ da,
                                                            int B, int H) {
  __shared__ float red[8][16][17];
  const int t = threadIdx.x, l = t & 63, w = t >> 6;
  int ug, rg;
  xcd_tile((B + 15) / 16, ug, rg);
  const int j0 = ug * 16, r0 = rg * 16;
  const int K = 4 * H;
  const int kq = ((K + 255) / 256) * 32;
  const int k0 = w * kq, k1 = (k0 + kq) < K ? (k0 + kq) : K;
  const int cl = l & 15;
  const bf16_t* brow = j0 + cl < H ? whh_t + (size_t)(j0 + cl) * K : nullptr;
  const bf16_t* arow = r0 + cl < B ? da_next + (size_t)(r0 + cl) * K : nullptr;
  // the element-wise operands of this thread's (row, unit) are requested before the product, not after it
  const int erow = (t >> 4) & 15, ecol = t & 15;
  const bool eok = t < 256 && r0 + erow < B && j0 + ecol < H;
  float ig = 0.f, fg = 0.f, gg = 0.f, og = 0.f, cc = 0.f, cp = 0.f, dcin = 0.f, dho = 0.f;
  if (eok) {
    const size_t idx = (size_t)(r0 + erow) * H + j0 + ecol, e0 = (size_t)(r0 + erow) * 4 * H + j0 + ecol;
    ig = gates[e0]; fg = gates[e0 + H]; gg = gates[e0 + 2 * H]; og = gates[e0 + 3 * H];
    cc = c[idx]; dcin = dc[idx];
    if (c_prev) cp = c_prev[idx];
    if (dh_out) dho = bf2f(dh_out[idx]);
  }
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  if (k0 < k1) wave_skinny_gemm16<16>(arow, brow, k0, k1, l, acc);  // 4H / 8 waves = 16 steps: one batch
#pragma unroll
  for (int r = 0; r < 4; ++r) red[w][4 * (l >> 4) + r][cl] = acc[r];
  __syncthreads();
  if (t < 256) {
    const int row = erow, col = ecol;
    const int b = r0 + row, j = j0 + col;
    if (eok) {
      float rec = 0.f;
#pragma unroll
      for (int q = 0; q < 8; ++q) rec += red[q][row][col];
      const size_t idx = (size_t)b * H + j;
      const float dh = dho + rec;
      const size_t e0 = (size_t)b * 4 * H + j;
      const float tc = tanhf(cc);
      const float dcv = dcin + dh * og * (1.f - tc * tc);
      da[e0] = f2bf(dcv * gg * ig * (1.f - ig));
      da[e0 + H] = f2bf(dcv * cp * fg * (1.f - fg));
      da[e0 + 2 * H] = f2bf(dcv * ig * (1.f - gg * gg));
      da[e0 + 3 * H] = f2bf(dh * tc * og * (1.f - og));
      dc[idx] = dcv * fg;
    }
  }
}


// ------------------------------------------------------------------------------------------------
// All time steps of a layer in ONE launch (forward, and the back-propagation through time).
// A workgroup owns 16 minibatch rows x 16 hidden units for the whole sequence and keeps its slice of the recurrent
// weights in LDS (forward: the 4 x 16 gate rows of W_hh, 64 x H; backward: 16 rows of W_hh^T, 16 x 4H) and its cell
// state / cell gradient in registers.  What the workgroups of one row group exchange per step is the hidden state
// (forward) or the gate gradients (backward) of those 16 rows, and the exchange is its own synchronisation: the
// launcher fills the sequence buffer with a pattern no result can have (bf16 0xffff, a NaN that f2bf_data never
// emits); producers write their 16 x 16 piece with agent-scope stores (through to memory instead of staying in the
// XCD's own L2); consumers fetch the 16-byte pieces they need with agent-scope loads and fetch again while any
// element still shows the pattern.  No counter, no fence, no cache-wide write-back or invalidate.  Measured with a
// stand-alone probe on MI355X (252 workgroups, values checked, no stale value in any run), per step: ordinary stores
// + device-scope fences 47 us; agent-scope stores, s_waitcnt, an arrival counter per row group and agent-scope loads
// 5.0 us (32 KB read per workgroup) to 6.4 us (126 KB); polling the data itself 4.7 us at 126 KB; a dependent launch
// per step costs about 8-10 us.  The grid must be resident at once: at most one workgroup per compute unit (the LDS
// slice sees to "at most"), grid <= number of compute units (the launcher checks).  EVERY WAIT IS BOUNDED: a wave that
// fetches `spin_limit` times without success, or sees the status word set, sets the status word and its workgroup
// leaves; the others follow, so the launch always ends.  The host reads the status word at its next
// synchronisation and reports the stage as failed.
// The arithmetic is that of the per-step kernels, in the same order (the waves split the reduction the same way and
// their partial tiles are added in wave order), so the results are bit-identical.
// ------------------------------------------------------------------------------------------------
typedef unsigned int seq_v4u __attribute__((ext_vector_type(4)));
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void seq_load16_agent(seq_v4u& dst, const void* p) {
  asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(dst) : "v"(p) : "memory");
}
#pragma clang diagnostic pop
__device__ __forceinline__ uint4 seq_u4(const seq_v4u& v) { return make_uint4(v.x, v.y, v.z, v.w); }

constexpr uint16_t kSeqEmpty = 0xffffu;  // what the launcher fills a sequence buffer with: "not written yet"
// bf16 rounding for exchanged data: never the "not written yet" pattern (a NaN whose payload would give it becomes the
// default NaN; finite values and infinities cannot collide with it)
__device__ __forceinline__ uint16_t f2bf_data(float v) {
  const uint16_t r = f2bf(v);
  return r == kSeqEmpty ? (uint16_t)0x7fc0u : r;
}
__device__ __forceinline__ bool seq_has_empty(const seq_v4u& v) {
  bool e = false;
#pragma unroll
  for (int i = 0; i < 4; ++i) e |= ((v[i] & 0xffffu) == 0xffffu) | ((v[i] >> 16) == 0xffffu);
  return e;
}
// One wave fetches its N pieces (lane addresses p[0..N)) until none of them shows the pattern.  false: gave up.
template <int N>
__device__ __forceinline__ bool seq_fetch(seq_v4u (&a)[N], const bf16_t* const (&p)[N], unsigned* status,
                                          unsigned spin_limit) {
  static_assert(N == 8, "the wait statement below names eight registers");
  unsigned spins = 0;
  for (;;) {
#pragma unroll
    for (int i = 0; i < N; ++i) seq_load16_agent(a[i], p[i]);
    asm volatile("s_waitcnt vmcnt(0)"
                 : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(a[4]), "+v"(a[5]), "+v"(a[6]), "+v"(a[7])
                 :
                 : "memory");
    bool miss = false;
#pragma unroll
    for (int i = 0; i < N; ++i) miss |= seq_has_empty(a[i]);
    if (!__any(miss)) return true;
    ++spins;
    if (spins > spin_limit ||
        ((spins & 63u) == 0u && __hip_atomic_load(status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u)) {
      __hip_atomic_store(status, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      return false;
    }
  }
}

constexpr int kSeqSettle = 12;  // s_sleep units (64 clocks each) before a forward step's first fetch
constexpr int kSeqMaxSteps = 8;  // reduction steps of 32 per wave: forward H <= 1024 on 4 waves

// sync[kSeqStatusWord]: the sticky status word.  starve: test hook -- the workgroups withhold what their peers wait
// for, so that no wait can succeed (and every one must still end).
__global__ __launch_bounds__(256, 1) void lstm_seq_fwd_kernel(float* __restrict__ gates, bf16_t* __restrict__ hbuf,
                                                              const bf16_t* __restrict__ whh,
                                                              float* __restrict__ cbuf, unsigned* __restrict__ sync,
                                                              int B, int H, int T, int row_bytes, unsigned spin_limit,
                                                              unsigned starve) {
  extern __shared__ __attribute__((aligned(16))) char seq_lds[];
  __shared__ float red[4][16][65];
  __shared__ uint16_t hs[16][16];
  __shared__ int give_up;
  const int t = threadIdx.x, l = t & 63, w = t >> 6;
  const int n_rg = (B + 15) / 16;
  const int rg = blockIdx.x % n_rg, ug = blockIdx.x / n_rg;
  const int u0 = ug * 16, r0 = rg * 16;
  unsigned* const status = sync + kSeqStatusWord;
  // W_hh slice -> LDS: row 16 q + u = gate q, unit u0 + u (zeros past H)
  {
    const int cpr = H / 8;  // 16-byte chunks per row
    for (int i = t; i < 64 * cpr; i += 256) {
      const int row = i / cpr, ch = i - row * cpr, q = row >> 4, u = u0 + (row & 15);
      const uint4 v = u < H ? ldg16(whh + ((size_t)q * H + u) * H + ch * 8) : zero16();
      *reinterpret_cast<uint4*>(seq_lds + (size_t)row * row_bytes + ch * 16) = v;
    }
  }
  if (t == 0) give_up = 0;
  __syncthreads();
  const int kq = ((H + 127) / 128) * 32;  // reduction elements per wave (as in the per-step kernel)
  const int k0 = w * kq, k1 = (k0 + kq) < H ? (k0 + kq) : H;
  const int cl = l & 15;
  const bool arow_ok = r0 + cl < B;
  const int erow = t >> 4, eu = t & 15;
  const bool eok = r0 + erow < B && u0 + eu < H;
  const size_t BH = (size_t)B * H;
  float cstate = eok ? cbuf[(size_t)(r0 + erow) * H + u0 + eu] : 0.f;  // c_{-1}
  for (int step = 0; step < T; ++step) {
    float gin[4] = {0.f, 0.f, 0.f, 0.f};
    if (eok) {
      const float* gp = gates + ((size_t)step * B + r0 + erow) * 4 * H + u0 + eu;
#pragma unroll
      for (int q = 0; q < 4; ++q) gin[q] = gp[(size_t)q * H];
    }
    f32x4 acc[4] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
    if (step > 0) {
      // Every lane fetches all of its pieces, from clamped addresses (what lies outside its share is zeroed below:
      // a load under a condition would leave the compiler free to copy the destination register at the end of the
      // conditional block, before the data has arrived); a clamped address is a piece some workgroup writes this step.
      const bf16_t* hrow = hbuf + (size_t)step * BH + (size_t)(arow_ok ? r0 + cl : B - 1) * H;  // h_{step-1}
      seq_v4u a[kSeqMaxSteps];
      const bf16_t* ap[kSeqMaxSteps];
#pragma unroll
      for (int st = 0; st < kSeqMaxSteps; ++st) {
        const int k = k0 + 32 * st + 8 * (l >> 4);
        ap[st] = hrow + (k < H - 8 ? k : H - 8);
      }
      // A first fetch right after this workgroup's own store comes too early for most of its peers' and costs a
      // whole round trip that also competes with their stores: wait about 0.4 us first (measured at H = 1000, 64
      // rows: 6.2 -> 5.3 us per step; the same pause in the backward kernel changes nothing).
      __builtin_amdgcn_s_sleep(kSeqSettle);
      if (!seq_fetch(a, ap, status, spin_limit)) give_up = 1;
      __syncthreads();
      if (give_up) return;
#pragma unroll
      for (int st = 0; st < kSeqMaxSteps; ++st) {
        const int k = k0 + 32 * st + 8 * (l >> 4);
        if (k0 + 32 * st < k1) {  // (wave-uniform)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const uint4 b = k < k1 ? *reinterpret_cast<const uint4*>(seq_lds + (size_t)(16 * q + cl) * row_bytes + k * 2)
                                   : zero16();
            const uint4 av = (k < k1 && arow_ok) ? seq_u4(a[st]) : zero16();
            acc[q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(frag(av), frag(b), acc[q], 0, 0, 0);
          }
        }
      }
    }
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
      for (int r = 0; r < 4; ++r) red[w][4 * (l >> 4) + r][16 * q + cl] = acc[q][r];
    __syncthreads();
    float hval = 0.f;
    if (eok) {
      float a4[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int col = 16 * q + eu;
        a4[q] = gin[q] + (((red[0][erow][col] + red[1][erow][col]) + red[2][erow][col]) + red[3][erow][col]);
      }
      const float ig = sigmoidf(a4[0]), fg = sigmoidf(a4[1]), gg = tanhf(a4[2]), og = sigmoidf(a4[3]);
      cstate = fg * cstate + ig * gg;
      float* gp = gates + ((size_t)step * B + r0 + erow) * 4 * H + u0 + eu;
      gp[0] = ig; gp[(size_t)H] = fg; gp[(size_t)2 * H] = gg; gp[(size_t)3 * H] = og;
      cbuf[(size_t)(step + 1) * BH + (size_t)(r0 + erow) * H + u0 + eu] = cstate;
      hval = og * tanhf(cstate);
    }
    hs[erow][eu] = f2bf_data(hval);
    __syncthreads();
    if (t < 128) {  // h_step -> memory, two units per lane, agent scope
      const int row = t >> 3, pr = t & 7, u = u0 + 2 * pr;
      if (r0 + row < B && u < H && !starve) {  // (H is even: units come in pairs)
        const uint32_t v = (uint32_t)hs[row][2 * pr] | ((uint32_t)hs[row][2 * pr + 1] << 16);
        uint32_t* dst = reinterpret_cast<uint32_t*>(hbuf + (size_t)(step + 1) * BH + (size_t)(r0 + row) * H + u);
        __hip_atomic_store(dst, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
    // (no wait: the next step's barriers order the LDS arrays, and nobody reads what this store overwrites)
  }
}

constexpr int kSeqMaxStepsBwd = 16;  // reduction steps of 32 per wave: 4H <= 4096 on 8 waves

__global__ __launch_bounds__(512, 1) void lstm_seq_bwd_kernel(const bf16_t* __restrict__ dh_out, bf16_t* __restrict__ dG,
                                                              const bf16_t* __restrict__ whh_t,
                                                              const float* __restrict__ gates,
                                                              const float* __restrict__ cbuf, unsigned* __restrict__ sync,
                                                              int B, int H, int T, int row_bytes, unsigned spin_limit,
                                                              unsigned starve) {
  extern __shared__ __attribute__((aligned(16))) char seq_lds[];
  __shared__ float red[8][16][17];
  __shared__ uint16_t das[16][4][16];
  __shared__ int give_up;
  const int t = threadIdx.x, l = t & 63, w = t >> 6;
  const int n_rg = (B + 15) / 16;
  const int rg = blockIdx.x % n_rg, ug = blockIdx.x / n_rg;
  const int j0 = ug * 16, r0 = rg * 16;
  const int K = 4 * H;
  unsigned* const status = sync + kSeqStatusWord;
  {  // W_hh^T slice -> LDS: row u = hidden unit j0 + u, 4H reduction elements (zeros past H)
    const int cpr = K / 8;
    for (int i = t; i < 16 * cpr; i += 512) {
      const int row = i / cpr, ch = i - row * cpr, u = j0 + row;
      const uint4 v = u < H ? ldg16(whh_t + (size_t)u * K + ch * 8) : zero16();
      *reinterpret_cast<uint4*>(seq_lds + (size_t)row * row_bytes + ch * 16) = v;
    }
  }
  if (t == 0) give_up = 0;
  __syncthreads();
  const int kq = ((K + 255) / 256) * 32;
  const int k0 = w * kq, k1 = (k0 + kq) < K ? (k0 + kq) : K;
  const int cl = l & 15;
  const bool arow_ok = r0 + cl < B;
  const int erow = (t >> 4) & 15, ecol = t & 15;
  const bool eok = t < 256 && r0 + erow < B && j0 + ecol < H;
  const size_t BH = (size_t)B * H;
  float dcs = 0.f;  // running dL/dc of this thread's (row, unit)
  for (int step = T - 1; step >= 0; --step) {
    float ig = 0.f, fg = 0.f, gg = 0.f, og = 0.f, cc = 0.f, cp = 0.f, dho = 0.f;
    if (eok) {
      const size_t idx = (size_t)(r0 + erow) * H + j0 + ecol;
      const float* gp = gates + ((size_t)step * B + r0 + erow) * 4 * H + j0 + ecol;
      ig = gp[0]; fg = gp[(size_t)H]; gg = gp[(size_t)2 * H]; og = gp[(size_t)3 * H];
      cc = cbuf[(size_t)(step + 1) * BH + idx];
      cp = cbuf[(size_t)step * BH + idx];
      if (dh_out) dho = bf2f(dh_out[(size_t)step * BH + idx]);
    }
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    if (step < T - 1) {
      const bf16_t* arow = dG + ((size_t)(step + 1) * B + (arow_ok ? r0 + cl : B - 1)) * K;  // da_{step+1}
      seq_v4u a[kSeqMaxStepsBwd];
      {  // two batches of eight pieces per lane (unconditional, clamped, as in the forward kernel)
        seq_v4u lo[8], hi[8];
        const bf16_t* plo[8];
        const bf16_t* phi[8];
#pragma unroll
        for (int st = 0; st < 8; ++st) {
          const int k = k0 + 32 * st + 8 * (l >> 4), k2 = k + 256;
          plo[st] = arow + (k < K - 8 ? k : K - 8);
          phi[st] = arow + (k2 < K - 8 ? k2 : K - 8);
        }
        if (!seq_fetch(lo, plo, status, spin_limit) || !seq_fetch(hi, phi, status, spin_limit)) give_up = 1;
#pragma unroll
        for (int st = 0; st < 8; ++st) { a[st] = lo[st]; a[8 + st] = hi[st]; }
      }
      __syncthreads();
      if (give_up) return;
#pragma unroll
      for (int st = 0; st < kSeqMaxStepsBwd; ++st) {
        const int k = k0 + 32 * st + 8 * (l >> 4);
        if (k0 + 32 * st < k1) {
          const uint4 b = k < k1 ? *reinterpret_cast<const uint4*>(seq_lds + (size_t)cl * row_bytes + k * 2) : zero16();
          const uint4 av = (k < k1 && arow_ok) ? seq_u4(a[st]) : zero16();
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(frag(av), frag(b), acc, 0, 0, 0);
        }
      }
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) red[w][4 * (l >> 4) + r][cl] = acc[r];
    __syncthreads();
    if (t < 256) {
      float d[4] = {0.f, 0.f, 0.f, 0.f};
      if (eok) {
        float rec = 0.f;
#pragma unroll
        for (int q = 0; q < 8; ++q) rec += red[q][erow][ecol];
        const float dh = step < T - 1 ? dho + rec : dho;  // (the last step has no recurrent term: keep a -0 as it is)
        const float tc = tanhf(cc);
        const float dcv = dcs + dh * og * (1.f - tc * tc);
        d[0] = dcv * gg * ig * (1.f - ig);
        d[1] = dcv * cp * fg * (1.f - fg);
        d[2] = dcv * ig * (1.f - gg * gg);
        d[3] = dh * tc * og * (1.f - og);
        dcs = dcv * fg;
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) das[erow][q][ecol] = f2bf_data(d[q]);
    }
    __syncthreads();
    {  // da_step -> memory: 16 rows x 4 gates x 8 pairs of units = 512 words, one per thread, agent scope
      const int row = t >> 5, q = (t >> 3) & 3, pr = t & 7, u = j0 + 2 * pr;
      if (r0 + row < B && u < H && !starve) {
        const uint32_t v = (uint32_t)das[row][q][2 * pr] | ((uint32_t)das[row][q][2 * pr + 1] << 16);
        uint32_t* dst = reinterpret_cast<uint32_t*>(dG + ((size_t)step * B + r0 + row) * K + (size_t)q * H + u);
        __hip_atomic_store(dst, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
  }
}

// LDS row stride for a slice whose rows hold `row_data_bytes`: padded so that 16 consecutive rows, read 16 bytes per
// lane at one reduction offset, fall into 16 different groups of four banks (stride = 16 mod 256 bytes)
int seq_row_bytes(int row_data_bytes) { return row_data_bytes + ((16 - row_data_bytes % 256) + 256) % 256; }
constexpr size_t kSeqLdsLimit = 160 * 1024 - 18 * 1024;  // what the kernels' static arrays leave of a compute unit's LDS

}  // namespace

hipError_t lstm_cell_forward(hipStream_t s, float* gates, const float* rec_part, int splits, const float* c_prev, float* c,
                             bf16_t* h, int B, int H) {
  lstm_cell_fwd_kernel<<<(B * H + 255) / 256, 256, 0, s>>>(gates, rec_part, rec_part ? splits : 0, c_prev, c, h, B, H);
  return hipGetLastError();
}

hipError_t lstm_cell_backward(hipStream_t s, const bf16_t* dh_out, const float* rec_part, int splits, float* dc,
                              const float* gates, const float* c, const float* c_prev, bf16_t* da, int B, int H) {
  lstm_cell_bwd_kernel<<<(B * H + 255) / 256, 256, 0, s>>>(dh_out, rec_part, rec_part ? splits : 0, dc, gates, c, c_prev,
                                                            da, B, H);
  return hipGetLastError();
}

hipError_t lstm_step_forward(hipStream_t s, float* gates, const bf16_t* h_prev, const bf16_t* whh, const float* c_prev,
                             float* c, bf16_t* h, int B, int H) {
  if ((H % 8) || !h_prev) return hipErrorInvalidValue;
  lstm_step_fwd_kernel<<<((H + 3) / 4) * ((B + 15) / 16), 256, 0, s>>>(gates, h_prev, whh, c_prev, c, h, B, H);
  return hipGetLastError();
}

hipError_t lstm_step_backward(hipStream_t s, const bf16_t* dh_out, const bf16_t* da_next, const bf16_t* whh_t, float* dc,
                              const float* gates, const float* c, const float* c_prev, bf16_t* da, int B, int H) {
  if ((H % 8) || !da_next) return hipErrorInvalidValue;
  lstm_step_bwd_kernel<<<((H + 15) / 16) * ((B + 15) / 16), 512, 0, s>>>(dh_out, da_next, whh_t, dc, gates, c, c_prev,
                                                                       da, B, H);
  return hipGetLastError();
}


// The multi-step kernels apply when the whole grid (one 16 x 16 tile of rows x units per workgroup) is resident at
// once and a workgroup's slice of the recurrent weights fits into LDS.
bool lstm_seq_applies(int B, int H, int T, int n_cus) {
  if (T < 2 || (H % 8) != 0 || H > 1024 || B < 1) return false;
  const int n_rg = (B + 15) / 16, n_ug = (H + 15) / 16;
  if (n_rg * n_ug > n_cus || ((size_t)B * H) % 8 != 0) return false;  // (the pattern fill works in 16-byte pieces)
  return (size_t)64 * seq_row_bytes(2 * H) <= kSeqLdsLimit && (size_t)16 * seq_row_bytes(8 * H) <= kSeqLdsLimit;
}

static hipError_t seq_prepare(const void* kernel) {
  static std::mutex mu;
  static std::set<std::pair<int, const void*>> done;  // (device, kernel): dynamic LDS above the default limit allowed
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  std::lock_guard<std::mutex> g(mu);
  if (!done.count({dev, kernel})) {
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kSeqLdsLimit);
    if (e != hipSuccess) return e;
    done.insert({dev, kernel});
  }
  return hipSuccess;
}

hipError_t lstm_seq_forward(hipStream_t s, float* gates, bf16_t* hbuf, const bf16_t* whh, float* cbuf, unsigned* sync,
                            int B, int H, int T, unsigned spin_limit, unsigned starve) {
  const int n_rg = (B + 15) / 16, n_ug = (H + 15) / 16, rb = seq_row_bytes(2 * H);
  const size_t lds = (size_t)64 * rb;
  hipError_t e = seq_prepare(reinterpret_cast<const void*>(&lstm_seq_fwd_kernel));
  if (e != hipSuccess) return e;
  // h_0 .. h_{T-1} (behind the initial state) = "not written yet"
  e = fill_pattern16(s, hbuf + (size_t)B * H, (size_t)T * B * H * sizeof(bf16_t), 0xffffffffu);
  if (e != hipSuccess) return e;
  lstm_seq_fwd_kernel<<<n_rg * n_ug, 256, lds, s>>>(gates, hbuf, whh, cbuf, sync, B, H, T, rb, spin_limit, starve);
  return hipGetLastError();
}

hipError_t lstm_seq_backward(hipStream_t s, const bf16_t* dh_out, bf16_t* dG, const bf16_t* whh_t, const float* gates,
                             const float* cbuf, unsigned* sync, int B, int H, int T, unsigned spin_limit,
                             unsigned starve) {
  const int n_rg = (B + 15) / 16, n_ug = (H + 15) / 16, rb = seq_row_bytes(8 * H);
  const size_t lds = (size_t)16 * rb;
  hipError_t e = seq_prepare(reinterpret_cast<const void*>(&lstm_seq_bwd_kernel));
  if (e != hipSuccess) return e;
  e = fill_pattern16(s, dG, (size_t)T * B * 4 * H * sizeof(bf16_t), 0xffffffffu);
  if (e != hipSuccess) return e;
  lstm_seq_bwd_kernel<<<n_rg * n_ug, 512, lds, s>>>(dh_out, dG, whh_t, gates, cbuf, sync, B, H, T, rb, spin_limit, starve);
  return hipGetLastError();
}

}  // namespace pd
