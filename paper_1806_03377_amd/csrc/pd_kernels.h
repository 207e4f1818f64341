// Launchers of the HIP kernels behind the stage runtime.  Every launcher only enqueues on the
// given stream; none allocates, synchronises or memsets.  All pointers are device pointers.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace pd {

typedef uint16_t bf16_t;  // raw bfloat16 bits

// The step applied to a parameter w with gradient g and its one state value s (Section 5.1 names the optimisers):
//   kind 0, momentum SGD:  s <- a s + g ;            w <- w - lr s
//   kind 1, RMSProp:       s <- a s + (1 - a) g^2 ;  w <- w - lr g / (sqrt(s) + eps)
//   kind 2, gradient only: the kernel stores g where it would have stored w and touches neither the state nor
//           the bf16 ring copy (their pointers are still read, so they must be valid).  Used by replicated stages,
//           whose gradients are summed over the replicas before the step (replica_sum_update below).
struct UpdateRule {
  float lr, a, eps;
  int kind;
};
constexpr int kRuleGradOnly = 2;
constexpr int kMaxReplicas = 8;
// (the rule as a compile-time constant, for kernels whose inner loop should not carry the choice)
template <int KIND>
__host__ __device__ __forceinline__ void apply_update_as(const UpdateRule& u, float g, float& s, float& w) {
  if (KIND == 0) {
    s = u.a * s + g;
    w -= u.lr * s;
  } else {
    s = u.a * s + (1.f - u.a) * g * g;
    w -= u.lr * g / (sqrtf(s) + u.eps);
  }
}
__host__ __device__ __forceinline__ void apply_update(const UpdateRule& u, float g, float& s, float& w) {
  if (u.kind == 0) apply_update_as<0>(u, g, s, w);
  else apply_update_as<1>(u, g, s, w);
}

// ---- bf16 x bf16 -> fp32-accumulate MFMA GEMMs (gemm_bf16.hip) ---------------------------------
// Bytes of split-K scratch the fwd/dgrad launchers may use for this shape.
size_t gemm_bf16_workspace_bytes(int M, int N, int K);
// y[M][N] = act(x[M][K] * w[N][K]^T + b[N]); written as bf16 to y, or unrounded as fp32 to y_f32 if that is
// not null (then y is not written).
hipError_t linear_fwd_bf16(hipStream_t s, const bf16_t* x, const bf16_t* w, const bf16_t* b, bf16_t* y, float* y_f32,
                           int M, int N, int K, bool relu, float* ws, size_t ws_bytes);
// dx[M][K] = (dz[M][N] * w[N][K]) .* (mask[M][K] > 0)   (mask may be null); dx bf16.
hipError_t linear_dgrad_bf16(hipStream_t s, const bf16_t* dz, const bf16_t* w, const bf16_t* mask, bf16_t* dx, int M,
                             int N, int K, float* ws, size_t ws_bytes);
// Output tiles (256 x 256) from which forward/dgrad go to the compute-bound kernels below (default 128: half the
// chip's compute units); returns the previous value, values < 1 only query.
int set_big_tile_threshold(int min_tiles);
// Variant of the large-tile forward product: 0 = chosen by reduction length (the default); 4 = four waves of 128 x 128
// outputs; 8 = eight waves of 128 x 64; 104 / 108 = the same with 64-byte instead of 128-byte LDS tile rows.  Returns the
// old value in the same encoding.
int set_big_gemm_waves(int waves);
// Compute-bound versions for many rows (gemm_big_bf16.hip; 256 x 256 tiles, no split-K, no workspace):
//   fwd: y = act(x w^T + b) (x row stride ldx; bf16 y or fp32 y_f32);  dgrad: dx = (dz w) .* mask;
//   wgrad: dw[N][K] = dz^T x as fp32, db[N] = column sums of dz (db may be null).
// splits > 1: the reduction is split that many ways and the fp32 partial products go to part[splits][M][N] (b, y, y_f32,
// relu are then not used; the caller adds the parts up); hipErrorInvalidValue if the shape does not allow it.
hipError_t linear_fwd_big_bf16(hipStream_t s, const bf16_t* x, int ldx, const bf16_t* w, const bf16_t* b, bf16_t* y,
                               float* y_f32, int M, int N, int K, bool relu, int splits, float* part);
// dgrad and wgrad read an operand sideways; given scratch of the stated size they transpose it first (faster).
size_t linear_dgrad_big_scratch_bytes(int N, int K);
size_t linear_wgrad_big_scratch_bytes(int M, int N, int K);
// scratch that lets linear_wgrad_update_big_bf16 split the rows of a product with few output tiles (0: no split)
size_t linear_wgrad_update_big_scratch_bytes(int M, int N, int K);
hipError_t linear_dgrad_big_bf16(hipStream_t s, const bf16_t* dz, const bf16_t* w, const bf16_t* mask, bf16_t* dx, int M,
                                 int N, int K, void* scratch, size_t scratch_bytes, int splits);
hipError_t linear_wgrad_big_bf16(hipStream_t s, const bf16_t* dz, const bf16_t* x, float* dw, float* db, int M, int N,
                                 int K, void* scratch, size_t scratch_bytes);

// The weight gradient of a many-row product fused with the momentum-SGD step: g = dz^T x (+ column sums of dz for
// the bias); m <- mu*m + g; master <- master - lr*m; ring <- bf16(master).  `part` (N*K + N floats) receives g only
// when the fused kernel does not apply (odd sizes or alignment); the bias gradient always passes through part + N*K.
// master_b may be null (no bias).  scratch as for linear_wgrad_big_bf16.
hipError_t linear_wgrad_update_big_bf16(hipStream_t s, const bf16_t* dz, const bf16_t* x, float* part, int M, int N,
                                        int K, float* master_w, float* mom_w, bf16_t* ring_w, float* master_b,
                                        float* mom_b, bf16_t* ring_b, UpdateRule rule, void* scratch,
                                        size_t scratch_bytes);

// out[M][C] = a[M][R] * w as fp32 PARTIAL sums ws[split][M][C] (no epilogue): the caller's own kernel adds them
// in split order.  a has row stride lda; w is [C][R] (w_rows_are_reduction = false) or [R][C] (true).
hipError_t gemm_partial_bf16(hipStream_t s, bool w_rows_are_reduction, const bf16_t* a, int lda, const bf16_t* w, int M,
                             int C, int R, float* ws, size_t ws_bytes, int* splits_out);

// Weight gradient fused with the momentum-SGD update, for up to kMaxWgradLayers Linear layers in ONE launch:
// per layer g = dz[M][N]^T x[M][K]; m <- mu*m + g; master <- master - lr*m; ring <- bf16(master); the same
// for the bias with g_b = column sums of dz (master_b may be null to skip the bias).
constexpr int kMaxWgradLayers = 8;
struct WgradLayer {
  const bf16_t* dz;  // [M][N]
  const bf16_t* x;   // [M][K]
  float* master_w;   // [N][K]
  float* mom_w;
  bf16_t* ring_w;
  // both non-null: the master weights are not read from / written to master_w but kept as the previous ring copy
  // (ring_in, read) plus 16-bit remainders (rem_w, read and written): 16 instead of 18 bytes per parameter.  All
  // layers of a batch must agree.  The bias keeps its fp32 master.
  const bf16_t* ring_in;
  uint16_t* rem_w;
  float* master_b;   // [N] or null
  float* mom_b;
  bf16_t* ring_b;
  int M, N, K;        // M = rows reduced over (0: use the batch's M)
  unsigned tile_end;  // filled in by the launcher
};
struct WgradBatch {
  WgradLayer layer[kMaxWgradLayers];
  int count, M;
  UpdateRule rule;
};
hipError_t linear_wgrad_update_bf16(hipStream_t s, const WgradBatch& batch);
// fp32 master <-> (bf16 ring copy, 16-bit remainder), n elements (misc_kernels.hip); see master_split1 in bf16_util.h
hipError_t master_split(hipStream_t s, const float* master, bf16_t* ring, uint16_t* rem, size_t n);
hipError_t master_merge(hipStream_t s, const bf16_t* ring, const uint16_t* rem, float* master, size_t n);

// ---- bf16 convolution and pooling, NHWC (conv_bf16.hip) ------------------------------------------------
struct ConvGeom {
  int N, H, W, Ci;   // input  [N][H][W][Ci]
  int Ho, Wo, Co;    // output [N][Ho][Wo][Co]
  int kh, kw, stride, ph, pw;
  int up;            // > 1: the input is read as if zero-upsampled by this factor (logical size (H-1)*up+1 by
                     // (W-1)*up+1, data only at multiples of `up`); 0 or 1: plain.  Used by the gradient of a
                     // strided convolution.
};
struct ConvEpilogue {
  const bf16_t* bias;  // [Co] or null
  const bf16_t* mask;  // same shape as out: value kept where mask > 0; or null
  int relu;
  bf16_t* out;
};
// 3 x 3, stride 1, pad 1 with Ci a multiple of 64: the kernel that keeps a tile's input with its halo in LDS
// (conv_halo_bf16.hip); conv_forward_bf16 / conv_dgrad_bf16 dispatch to it.  set_conv_halo(0 / 1 / 2) switches it off / on / on without the weights-resident variant
// (returns the previous setting; any other argument only queries).
bool conv3x3_halo_applies(const ConvGeom& g, const bf16_t* x, const bf16_t* w);
hipError_t conv3x3_halo_bf16(hipStream_t s, const bf16_t* x, const bf16_t* w, const ConvGeom& g, const ConvEpilogue& ep);
int set_conv_halo(int on);
// kh*kw*Ci <= 32 and Co <= 64 (first layer of an image network): handled by the gather kernels
bool conv_is_smallk(const ConvGeom& g);
// The two kernels of that case (conv_smallk_bf16.hip); conv_forward_bf16 / conv_wgrad_partial_bf16 dispatch to them.
hipError_t conv_smallk_forward_bf16(hipStream_t s, const bf16_t* x, const bf16_t* w, const ConvGeom& g,
                                    const ConvEpilogue& ep);
hipError_t conv_smallk_wgrad_partial_bf16(hipStream_t s, const bf16_t* dz, const bf16_t* x, float* part, int splits,
                                          const ConvGeom& g);
// y = act(conv(x, w) + b); w[Co][kh][kw][Ci].  Needs Ci % 8 == 0 unless conv_is_smallk.
hipError_t conv_forward_bf16(hipStream_t s, const bf16_t* x, const bf16_t* w, const ConvGeom& g,
                             const ConvEpilogue& ep);
// dx = convT(dz, w) .* mask; wt_scratch holds Co*kh*kw*Ci elements (flipped, transposed weights).  For stride s > 1
// the transposed convolution reads dz zero-upsampled by s (taps that fall between samples contribute nothing).
hipError_t conv_dgrad_bf16(hipStream_t s, const bf16_t* dz, const bf16_t* w, bf16_t* wt_scratch, const ConvGeom& g,
                           const ConvEpilogue& ep);
// Output tiles (256 x 256) from which forward / input-gradient convolutions with >= 256 output channels use the
// wide-tile kernel (default 256: one tile per compute unit).
void set_conv_wide_min_tiles(int min_tiles);
// Number of partial sums the weight-gradient kernel produces for this geometry, and the kernel itself:
// part[split][Co*kh*kw*Ci + Co] (weights in w's layout, then the bias gradient).
int conv_wgrad_split_count(const ConvGeom& g);
hipError_t conv_wgrad_partial_bf16(hipStream_t s, const bf16_t* dz, const bf16_t* x, float* part, int splits,
                                   const ConvGeom& g);
// The same partial sums for stride-1 convolutions with at most "same" padding (conv_wgrad_tr_bf16.hip: all taps of a group of
// filter rows in one workgroup, operands fetched with transposing LDS reads).  conv_wgrad_tr_partials returns the
// number of partials that kernel writes for this geometry, or 0 if the geometry is not covered;
// conv_wgrad_split_count / conv_wgrad_partial_bf16 above choose between the two kernels themselves.
int conv_wgrad_tr_partials(const ConvGeom& g);
hipError_t conv_wgrad_tr_partial_bf16(hipStream_t s, const bf16_t* dz, const bf16_t* x, float* part, int partials,
                                      const ConvGeom& g);
// g = sum of the partials in split order; m <- mu*m + g; master <- master - lr*m; ring <- bf16(master).
// Partial s starts at part + s*stride (stride 0 = n_w + n_b); n_b may be 0 to leave the bias alone.
hipError_t wgrad_reduce_update(hipStream_t s, const float* part, int splits, size_t stride, size_t n_w, int n_b,
                               float* master_w, float* mom_w, bf16_t* ring_w, float* master_b, float* mom_b,
                               bf16_t* ring_b, UpdateRule rule);
// General pooling over NHWC (window k x k, stride, zero padding `pad` on every side; C % 8 == 0):
//   max: padding never wins; backward sends dy to the FIRST maximum of each window in row-major order and sums,
//        per input position, the contributions of the windows that cover it in row-major window order
//   avg: sum of the window (padding counts as zeros) divided by k*k; backward = the transposed operator
// relu_mask (backward): additionally zero dx where x <= 0.
struct PoolGeom {
  int N, H, W, C, k, stride, pad, Ho, Wo;
};
// route (max pooling with a window of at most 4, else it must be null): null, or N * Ho * Wo * C bytes (8-byte
// aligned) that record where each maximum came from; pool2d_backward_routed_bf16 then needs neither x nor y
bool pool2d_routes(bool is_max, const PoolGeom& g);
hipError_t pool2d_forward_bf16(hipStream_t s, bool is_max, const bf16_t* x, bf16_t* y, void* route, const PoolGeom& g);
hipError_t pool2d_backward_routed_bf16(hipStream_t s, const void* route, const bf16_t* dy, bf16_t* dx, const PoolGeom& g,
                                       bool relu_mask);
hipError_t pool2d_backward_bf16(hipStream_t s, bool is_max, const bf16_t* x, const bf16_t* y, const bf16_t* dy,
                                bf16_t* dx, const PoolGeom& g, bool relu_mask);
// Channel concatenation helpers for [pixels][channels] bf16 tensors (all channel counts % 8 == 0):
//   copy_channels: dst[p][dst_off .. dst_off+c) = src[p][src_off .. src_off+c)   (row strides ld_dst, ld_src);
//                  with mask != null (same layout as dst) values are zeroed where mask <= 0
//   sum_tensors:   dst = bf16(sum_i src[i]) in index order (fp32), times (mask > 0) if mask != null; n elements
hipError_t copy_channels_bf16(hipStream_t s, const bf16_t* src, int ld_src, int src_off, bf16_t* dst, int ld_dst,
                              int dst_off, const bf16_t* mask, size_t pixels, int c);
constexpr int kMaxBranches = 8;
hipError_t sum_tensors_bf16(hipStream_t s, const bf16_t* const* src, int count, const bf16_t* mask, bf16_t* dst,
                            size_t n);
// route: null, or N * (H/2) * (W/2) * (C/8) words that record where each maximum came from (four bits per output
// element); maxpool2x2_backward_routed_bf16 then needs neither x nor y
hipError_t maxpool2x2_forward_bf16(hipStream_t s, const bf16_t* x, bf16_t* y, uint32_t* route, int N, int H, int W,
                                   int C);
hipError_t maxpool2x2_backward_routed_bf16(hipStream_t s, const uint32_t* route, const bf16_t* dy, bf16_t* dx, int N,
                                           int H, int W, int C, bool relu_mask);
// dx = dy routed to the first maximum of each window (row-major), times (x > 0) if relu_mask
hipError_t maxpool2x2_backward_bf16(hipStream_t s, const bf16_t* x, const bf16_t* y, const bf16_t* dy, bf16_t* dx, int N,
                                    int H, int W, int C, bool relu_mask);

// ---- LSTM cell kernels (lstm_bf16.hip); gate order i, f, g, o; all [B][.] row-major ---------------------------
// gates <- act(gates + sum_s rec_part[s]) in place (gates holds x_t W_ih^T + b on entry; rec_part may be null);
// c <- f*c_prev + i*g; h <- bf16(o*tanh(c)).
hipError_t lstm_cell_forward(hipStream_t s, float* gates, const float* rec_part, int splits, const float* c_prev, float* c,
                             bf16_t* h, int B, int H);
// One step of back-propagation through time: dh = dh_out + sum_s rec_part[s] (either may be null), dc updated
// in place (on exit dL/dc_{t-1}), da[B][4H] = bf16 gradient w.r.t. the gate pre-activations.
hipError_t lstm_cell_backward(hipStream_t s, const bf16_t* dh_out, const float* rec_part, int splits, float* dc,
                              const float* gates, const float* c, const float* c_prev, bf16_t* da, int B, int H);

// The same two steps with the recurrent product fused in (one launch per time step):
//   forward : gates += h_prev[B][H] * whh[4H][H]^T, then as lstm_cell_forward        (h_prev not null)
//   backward: dh = dh_out + da_next[B][4H] * whh_t[H][4H]^T, then as lstm_cell_backward  (da_next not null)
// The whole sequence of a layer in one launch (see lstm_bf16.hip).  sync: kSeqSyncWords device words owned by the
// stage; word kSeqStatusWord is the sticky status (non-zero = a workgroup gave up waiting).  The launchers first fill
// the part of hbuf / dG that the launch produces with the "not written yet" pattern.  starve: test hook (no workgroup
// publishes its results, so no wait can succeed).
constexpr int kSeqStatusWord = 16, kSeqSyncWords = 32;
bool lstm_seq_applies(int B, int H, int T, int n_cus);
hipError_t lstm_seq_forward(hipStream_t s, float* gates, bf16_t* hbuf, const bf16_t* whh, float* cbuf, unsigned* sync,
                            int B, int H, int T, unsigned spin_limit, unsigned starve);
hipError_t lstm_seq_backward(hipStream_t s, const bf16_t* dh_out, bf16_t* dG, const bf16_t* whh_t, const float* gates,
                             const float* cbuf, unsigned* sync, int B, int H, int T, unsigned spin_limit,
                             unsigned starve);
hipError_t lstm_step_forward(hipStream_t s, float* gates, const bf16_t* h_prev, const bf16_t* whh, const float* c_prev,
                             float* c, bf16_t* h, int B, int H);
hipError_t lstm_step_backward(hipStream_t s, const bf16_t* dh_out, const bf16_t* da_next, const bf16_t* whh_t, float* dc,
                              const float* gates, const float* c, const float* c_prev, bf16_t* da, int B, int H);

// ---- update of a replicated stage (update.hip) ---------------------------------------------------
// g = grads.g[0] + grads.g[1] + ... (in that order), then the step of `rule` on (w_in -> w_out, state) and
// ring <- bf16(w_out) if ring is not null.  All arrays 16-byte aligned, n elements each.
struct ReplicaGrads {
  const float* g[kMaxReplicas];
  int count;
};
hipError_t replica_sum_update(hipStream_t s, const ReplicaGrads& grads, const float* w_in, float* w_out, float* state,
                              bf16_t* ring, size_t n, UpdateRule rule);

// ---- fp32 path (linear_f32.hip) ------------------------------------------------------------------
hipError_t linear_fwd_f32(hipStream_t s, const float* x, const float* w, const float* b, float* y, int M, int N, int K,
                          bool relu);
hipError_t linear_dgrad_f32(hipStream_t s, const float* dz, const float* w, const float* mask, float* dx, int M, int N,
                            int K);
// w_out <- w_in - lr*(m <- mu*m + dz^T x); w_in may equal w_out.
hipError_t linear_wgrad_update_f32(hipStream_t s, const float* dz, const float* x, const float* w_in, float* w_out,
                                   float* mom_w, const float* b_in, float* b_out, float* mom_b, int M, int N, int K,
                                   UpdateRule rule);

// ---- element-wise and loss kernels (misc_kernels.hip) --------------------------------------------
hipError_t copy_bytes(hipStream_t s, const void* src, void* dst, size_t bytes);  // bytes % 4 == 0 or any
hipError_t fill_zero(hipStream_t s, void* dst, size_t bytes);
// every 32-bit word of dst[0 .. bytes) = value; dst 16-byte aligned, bytes a multiple of 16
hipError_t fill_pattern16(hipStream_t s, void* dst, size_t bytes, uint32_t value);
hipError_t f32_to_bf16(hipStream_t s, const float* src, bf16_t* dst, size_t n);
hipError_t transpose_bf16(hipStream_t s, const bf16_t* src, bf16_t* dst, int R, int C);  // dst[C][R] = src[R][C]^T
hipError_t bf16_to_f32(hipStream_t s, const bf16_t* src, float* dst, size_t n);
// dz = dy .* (y > 0)   (bf16 or fp32 elements, n elements)
hipError_t relu_mask(hipStream_t s, const void* dy, const void* y, void* dz, size_t n, bool is_bf16);
// softmax cross-entropy over rows: dlogits = (softmax - onehot)/rows, row_loss[r] = -log softmax[label];
// then *loss = mean(row_loss) (summed in row order by one workgroup).  loss may be null.
// logits are always fp32; dlogits are bf16 if dlogits_bf16, else fp32.
hipError_t softmax_xent(hipStream_t s, const float* logits, const int32_t* labels, void* dlogits, float* row_loss,
                        float* loss, int rows, int classes, bool dlogits_bf16);
// The same when the logits still are split-K partial sums part[split][rows][classes] (+ bias[classes], may be null):
// adds them up in split order, writes the fp32 logits once, and takes the loss from registers.  classes <=
// kFusedLossMaxClasses.
constexpr int kFusedLossMaxClasses = 2048;
hipError_t softmax_xent_partials(hipStream_t s, const float* part, int splits, const bf16_t* bias, float* logits,
                                 const int32_t* labels, void* dlogits, float* row_loss, float* loss, int rows,
                                 int classes, bool dlogits_bf16);
// Whether linear_fwd_bf16 would hand this shape to the compute-bound large-tile kernel (which has no split-K).
bool linear_fwd_uses_big_tiles(int M, int N);

}  // namespace pd
