// Host side of the stage runtime: the C ABI of include/pd.h.
//
// Holds only integers and pointers: the static 1F1B op list (Section 3.3), the weight-version ring and
// the per-minibatch stash table (Sections 3.4 and 4), the carving of the caller's arena (Section 3.5),
// and the enqueue order of the HIP kernels.  No arithmetic of the method happens on the host.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>

#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <deque>
#include <new>
#include <string>
#include <map>
#include <mutex>
#include <vector>

#include "../../include/pd.h"
#include "../../include/pd_debug.h"
#include "pd_error.h"
#include "pd_kernels.h"

namespace {
thread_local std::string g_err;
}

namespace pd {
int fail(int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_err = buf;
  return code;
}
}  // namespace pd

namespace {
using pd::fail;

#define PD_HIP(expr)                                                                           \
  do {                                                                                         \
    hipError_t e_ = (expr);                                                                    \
    if (e_ != hipSuccess) return fail(PD_EHIP, "%s: %s", #expr, hipGetErrorString(e_));        \
  } while (0)

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---- schedule ------------------------------------------------------------------------------------
// Start-up forwards, then for every minibatch k in arrival order: its backward, its update, and the
// forward that refills the slot it freed.  `latest` is carried along exactly as the stage does.
void build_schedule(int depth, int M, std::vector<pd_op>& ops) {
  ops.clear();
  if (M <= 0) return;
  const int W = depth < M ? depth : M;  // a short stream never fills the stage
  std::vector<int> seen(M, 0);
  int latest = 0;
  for (int i = 0; i < W; ++i) {
    seen[i] = latest;
    ops.push_back({PD_OP_F, i, latest, latest % depth});
  }
  for (int k = 0; k < M; ++k) {
    ops.push_back({PD_OP_B, k, seen[k], seen[k] % depth});
    ++latest;
    ops.push_back({PD_OP_U, k, latest, latest % depth});
    const int nf = k + W;
    if (nf < M) {
      seen[nf] = latest;
      ops.push_back({PD_OP_F, nf, latest, latest % depth});
    }
  }
}

int stage_depth(int num_stages, int noam, int stage_index) {
  (void)num_stages;
  const int d = noam - stage_index;
  return d < 1 ? 1 : d;
}

int emit_schedule(int depth, int M, pd_op* out, size_t cap, size_t* n_out) {
  std::vector<pd_op> ops;
  build_schedule(depth, M, ops);
  if (n_out) *n_out = ops.size();
  if (ops.size() > cap) return fail(PD_ENOMEM, "schedule needs %zu entries, capacity %zu", ops.size(), cap);
  if (!ops.empty()) {
    if (!out) return fail(PD_EINVAL, "out is null");
    memcpy(out, ops.data(), ops.size() * sizeof(pd_op));
  }
  return PD_OK;
}

enum { K_LINEAR = 0, K_CONV = 1, K_POOL = 2, K_LSTM = 3, K_GPOOL = 4, K_CONCAT = 5 };
// K_POOL: the 2x2/stride-2 max pooling fast path; K_GPOOL: any other max or average pooling; K_CONCAT: the
// channel concatenation that closes a block of parallel branches (a layer without parameters whose output is
// assembled from the branch outputs).

// From this many rows on, a Linear/LSTM weight gradient is formed by the large-reduction kernel (fp32 partial
// sums over row ranges, then a fused reduce + update) instead of the kernel built for minibatch-sized reductions.
constexpr int kBigRows = 512;

pd::ConvGeom rows_as_pixels(int rows, int k, int n) {  // y[rows][n] = x[rows][k] w[n][k]^T seen as a 1x1 convolution
  return pd::ConvGeom{rows, 1, 1, k, 1, 1, n, 1, 1, 1, 0, 0};
}

// One compute layer of the stage.  Activations are [minibatch][h][w][c] (NHWC); a Linear sees its input
// flattened in that order: in = ih*iw*ic, out = oc with oh = ow = 1.
struct Layer {
  int kind = K_LINEAR;
  int rows = 0;            // rows of the activation matrices: minibatch, or seq_len * minibatch after an LSTM
  int T = 1;               // LSTM: sequence length
  int in = 0, out = 0;     // features per row in / out
  int ih = 1, iw = 1, ic = 0, oh = 1, ow = 1, oc = 0;
  int kh = 1, kw = 1, stride = 1, ph = 0, pw = 0;
  bool relu = false;
  size_t n_w = 0, n_b = 0;     // parameter counts (0 for pooling)
  size_t w_off = 0, b_off = 0;    // element offsets inside one parameter set on the device (padded)
  size_t flat_w = 0, flat_b = 0;  // element offsets inside the caller's flat vector
  size_t y_off = 0;           // byte offset of this layer's output inside a stash slot
  size_t dz_off = 0;          // Linear: byte offset of dL/d(pre-activation) inside the gradient workspace
  size_t part_off = 0;        // conv: byte offset of the weight-gradient partial sums
  int splits = 0;             // conv: number of partial sums (also Linear/LSTM layers with many rows, see kBigRows)
  bool split_master = false;  // bf16 Linear/LSTM layers updated by the fused kernel: master = ring copy + remainder
  size_t part2_off = 0;       // LSTM with many rows: partial sums of the W_hh gradient
  int splits2 = 0;
  size_t g_off = 0, c_off = 0;  // LSTM: byte offsets inside a stash slot of the gate values [T][B][4H] fp32 and
                                // the cell states [T+1][B][H] fp32 (slot 0 = zeros); y_off holds [T+1][B][H] hidden
                                // states (slot 0 = zeros), the layer's output starts at slot 1
  size_t dc_off = 0;          // LSTM: byte offset of dL/dc [B][H] fp32 inside the gradient workspace
  // data flow: the layer whose stored output this layer reads (-1: the stage input).  In a chain that is the
  // layer before; the first layer of every branch of a block reads the block's input.
  int src = -1;
  bool is_max = false;        // K_GPOOL: max (true) or average pooling
  int block = -1;             // index of the K_CONCAT layer closing the block this layer is in (-1: none)
  bool br_first = false, br_last = false;
  size_t bdy_off = 0;         // last layer of a branch: where its slice of the block's output gradient is staged
  size_t bdx_off = 0;         // first layer of a branch: where its contribution to the block's input gradient goes
  // K_CONCAT: the branches (first and last layer, channel offset and count of each slice), the block's input
  int nbr = 0, b_first[pd::kMaxBranches] = {}, b_last[pd::kMaxBranches] = {}, b_coff[pd::kMaxBranches] = {},
      b_c[pd::kMaxBranches] = {};
  int blk_src = -1;
  size_t blk_in_elems = 0;    // elements of the block's input (rows * features)
};
typedef Layer Linear;  // (historic name used below for "a layer")

struct InFlight {
  int mb, version;
};

}  // namespace

struct pd_stage {
  int stage_index = 0, num_stages = 1, noam = 1;
  int depth = 1, in_depth = 1;
  int ring_depth = 1;        // weight versions kept: depth, or the input stage's depth under vertical sync
  bool vsync = false;
  int B = 0;
  bool bf16 = false;
  bool has_loss = false;
  int classes = 0;
  pd::UpdateRule rule = {0.f, 0.f, 0.f, 0};
  hipStream_t stream = nullptr;
  // Backward lane (cfg.stream_backward): the kernels of pd_backward run on stream_b, next to the update and the forward
  // pass that the 1F1B order places before them.  What pd_backward writes for pd_update (the factored gradient dz, the
  // convolutions' partial sums) exists twice and consecutive backward passes alternate between the two sets, so B(k+1)
  // only has to wait for U(k-1), the update that read the set it overwrites, not for U(k).
  //   ev_fwd[mb % depth]  that minibatch's forward pass on `stream` is done (B reads its stash slot)
  //   ev_upd[n & 1]       the n-th update on `stream` is done
  //   ev_bwd              the last backward pass on stream_b is done (the update reads what it wrote)
  //   ws_b                the lane's own split-K workspace
  hipStream_t stream_b = nullptr;
  hipEvent_t ev_upd[2] = {nullptr, nullptr}, ev_bwd = nullptr;
  std::vector<hipEvent_t> ev_fwd;
  long long n_upd = 0;       // updates enqueued so far
  int bwd_set = 0;           // which set of gradient buffers the next backward pass writes
  char *dz_base = nullptr, *part_base = nullptr;
  size_t dz_set_bytes = 0, part_set_bytes = 0;
  float* ws_b = nullptr;
  hipStream_t bstream() const { return stream_b ? stream_b : stream; }
  hipError_t sync_all() const {
    hipError_t e = hipStreamSynchronize(stream);
    if (e == hipSuccess && stream_b) e = hipStreamSynchronize(stream_b);
    return e;
  }
  std::vector<Linear> lin;
  size_t esz = 4;
  size_t n_params = 0;       // flat length
  size_t p_pad = 0;          // elements per parameter set on the device
  size_t in_bytes = 0, out_bytes = 0, stash_slot_bytes = 0, dlogits_off = 0;
  size_t pp_bytes = 0;       // one ping-pong gradient buffer of the conv/pool layers
  // device regions (inside the caller's arena)
  char* ring = nullptr;      // depth parameter sets (bf16 or fp32)
  float* master = nullptr;   // bf16 mode only
  // bf16 mode, unreplicated stages: the fp32 master weights of the layers with split_master set are NOT kept in
  // `master` but as the latest ring copy plus 16 low bits each in `rem` (see master_split1); `master` is then only
  // the staging area through which the host reads and writes them (materialize_master / split_master_from_staging)
  uint16_t* rem = nullptr;
  float* mom = nullptr;
  char* in_ring = nullptr;
  char* stash = nullptr;
  char* dz = nullptr;
  char* grad_in = nullptr;   // 2 slots, stages without a loss
  char* pp = nullptr;        // two ping-pong activation-gradient buffers (conv/pool layers)
  char* part = nullptr;      // conv weight-gradient partial sums, all layers
  char* wt = nullptr;        // flipped/transposed conv weights for dgrad (largest layer)
  char* blk_dy = nullptr;    // block backward: the output gradient split into per-branch contiguous tensors
  char* blk_dx = nullptr;    // block backward: one input-gradient tensor per branch, summed afterwards
  size_t blk_dx_stride = 0;
  float* ws = nullptr;
  size_t ws_bytes = 0;
  float* row_loss = nullptr;
  // multi-step recurrence kernels: arrival counters + sticky status word, one block for the forward and one for the
  // backward direction (with a backward stream the two can be in flight together)
  unsigned* seq_sync = nullptr;
  bool seq_used = false;     // a multi-step kernel has been enqueued since the status word was last read
  int n_cus = 0;
  // replicated stage (Section 3.3, Section 4 "Data Parallelism"): every replica is a pd_stage of its own (stash,
  // scratch, stream); ring, master and mom of a secondary replica point into the primary's arena, and each replica
  // leaves the fp32 gradient of its minibatch in gradbuf (laid out like one parameter set) for the summed update
  int n_replicas = 1;
  float* gradbuf = nullptr;
  pd_stage* primary = nullptr;          // null on the primary itself
  std::vector<pd_stage*> secondaries;   // primary only
  hipEvent_t ev_rep = nullptr;          // this replica's stream has reached the joint update / the update is done
  pd_stage_config cfg = {};
  std::vector<pd_layer_desc> cfg_layers;
  // protocol state
  int latest = 0;
  int last_fwd = -1;
  std::deque<InFlight> in_flight;
  bool grad_pending = false;
  int pending_mb = -1;
  // the most recent trace_cap executed ops (bounded: a stage may run for the whole of training)
  std::deque<pd_op> trace;
  size_t trace_cap = 65536;
  void log_op(int kind, int mb, int version) {
    if (!trace_cap) return;
    if (trace.size() >= trace_cap) trace.pop_front();
    trace.push_back({kind, mb, version, version % ring_depth});
  }
  // events of the pipeline drivers: rings indexed by minibatch (or round) modulo their length, which depends on
  // the in-flight depths only, never on the length of the stream; created on first use, reused by later calls
  std::vector<hipEvent_t> ev_f, ev_b, ev_u;
  // layer profiler (Section 3.2): while `profiling`, every op drops an event after each layer's kernels; the time
  // between two consecutive marks belongs to the layer named by the later one (the stream runs kernels in order)
  struct Mark { int phase, layer; hipEvent_t ev; };  // phase: -1 = start of an op, 0 F, 1 B, 2 U, 3 U of the batch
  bool profiling = false;
  std::vector<Mark> marks;
  std::vector<hipEvent_t> mark_pool;
  int prof_ops[3] = {0, 0, 0};
  hipError_t mark(int phase, int layer) {
    if (!profiling) return hipSuccess;
    hipEvent_t e;
    if (!mark_pool.empty()) { e = mark_pool.back(); mark_pool.pop_back(); }
    else { const hipError_t rc = hipEventCreate(&e); if (rc != hipSuccess) return rc; }
    marks.push_back({phase, layer, e});
    return hipEventRecord(e, stream);
  }

  // Zero-copy hand-off (pd_pipeline_run): per stash slot, where the LAST layer's output of the minibatch in that slot
  // lives when it was written straight into the consumer stage's input slot instead of the stash (null: in the stash);
  // and, until pd_update, where dL/d(pre-activation) of the last layer lies when the consumer stage has left it, masked,
  // in this stage's gradient slot (null: in the stage's own buffer)
  std::vector<char*> borrowed_out;
  const char* borrowed_dz = nullptr;

  char* ring_slot(int version) const { return ring + (size_t)(version % ring_depth) * p_pad * esz; }
  char* in_slot(int mb) const { return in_ring + (size_t)(mb % in_depth) * in_bytes; }
  char* stash_slot(int mb) const { return stash + (size_t)(mb % depth) * stash_slot_bytes; }
  char* grad_slot(int mb) const { return grad_in + (size_t)(mb & 1) * out_bytes; }
  // stored output of layer l inside a stash slot (an LSTM keeps a zero state in front of its sequence)
  char* out_of(char* slot, int l) const {
    const Linear& L = lin[l];
    if (l + 1 == (int)lin.size() && !borrowed_out.empty()) {
      char* b = borrowed_out[(size_t)(slot - stash) / stash_slot_bytes];
      if (b) return b;
    }
    return slot + L.y_off + (L.kind == K_LSTM ? (size_t)B * L.out * 2 : 0);
  }
};

namespace {

struct Plan {
  std::vector<Linear> lin;
  bool has_loss = false, bf16 = false;
  int classes = 0, depth = 1, in_depth = 1, ring_depth = 1, B = 0;
  size_t esz = 4, n_params = 0, p_pad = 0, in_bytes = 0, out_bytes = 0, stash_slot_bytes = 0, dlogits_off = 0;
  size_t ws_bytes = 0, dz_bytes = 0, pp_bytes = 0, part_bytes = 0, wt_bytes = 0;
  size_t blk_dy_bytes = 0, blk_dx_bytes = 0, blk_dx_stride = 0, o_blk_dy = 0, o_blk_dx = 0;
  // arena offsets
  size_t o_rem = 0;
  bool any_split = false;
  size_t o_ring = 0, o_master = 0, o_mom = 0, o_in = 0, o_stash = 0, o_dz = 0, o_grad = 0, o_ws = 0, o_rowloss = 0;
  size_t o_pp = 0, o_part = 0, o_wt = 0, o_gradbuf = 0, o_ws_b = 0, o_seq = 0;
  bool lane_b = false;
  int replicas = 1;
  size_t total = 0;
};

// secondary: lay out the arena of a further replica of a replicated stage (no parameter state of its own)
int make_plan(const pd_stage_config* c, Plan& p, bool secondary = false) {
  if (!c) return fail(PD_EINVAL, "config is null");
  if (c->replicas < 0 || c->replicas > pd::kMaxReplicas) return fail(PD_EINVAL, "replicas must be 0..%d (got %d)", pd::kMaxReplicas, c->replicas);
  p.replicas = c->replicas > 1 ? c->replicas : 1;
  if (p.replicas > 1 && c->vertical_sync) return fail(PD_EINVAL, "vertical sync is not available for a replicated stage");
  if (secondary && p.replicas < 2) return fail(PD_EINVAL, "the stage is not configured as replicated");
  p.lane_b = c->stream_backward != nullptr;
  if (p.lane_b && p.replicas > 1) return fail(PD_EINVAL, "a replicated stage cannot have a backward stream of its own");
  if (p.lane_b && c->stream_backward == c->stream) return fail(PD_EINVAL, "stream_backward must differ from stream (or be null)");
  if (c->optimizer != PD_OPT_SGD_MOMENTUM && c->optimizer != PD_OPT_RMSPROP) return fail(PD_EINVAL, "unknown optimizer %d", c->optimizer);
  if (c->optimizer == PD_OPT_RMSPROP && !(c->eps > 0.f)) return fail(PD_EINVAL, "RMSProp needs eps > 0");
  if (c->num_stages < 1 || c->stage_index < 0 || c->stage_index >= c->num_stages)
    return fail(PD_EINVAL, "stage_index %d outside [0, %d)", c->stage_index, c->num_stages);
  if (c->noam < 1) return fail(PD_EINVAL, "noam must be >= 1");
  if (c->minibatch < 1) return fail(PD_EINVAL, "minibatch must be >= 1");
  if (c->precision != PD_F32 && c->precision != PD_BF16_F32ACC) return fail(PD_EINVAL, "unknown precision");
  if (c->n_layers < 1 || !c->layers) return fail(PD_EINVAL, "no layers");
  p.bf16 = c->precision == PD_BF16_F32ACC;
  p.esz = p.bf16 ? 2 : 4;
  p.B = c->minibatch;
  p.depth = c->in_flight_override > 0 ? c->in_flight_override : stage_depth(c->num_stages, c->noam, c->stage_index);
  p.in_depth = c->stage_index > 0 ? p.depth + 1 : p.depth;
  // vertical sync (Section 3.4): a minibatch may ask for a version as old as the input stage's oldest
  p.ring_depth = c->vertical_sync ? (c->in_flight_override > 0 ? c->in_flight_override : stage_depth(c->num_stages, c->noam, 0))
                                  : p.depth;
  if (p.ring_depth < p.depth) p.ring_depth = p.depth;
  size_t flat = 0, dev = 0, y_off = 0, dz_off = 0, part_off = 0;
  int width = -1;               // features per row produced so far (-1: stage input not yet known)
  int ch = 0, hh = 1, ww = 1;   // its NHWC shape
  int rows = p.B;               // rows of the current activation matrix
  size_t x_off = 0;             // LSTM extras inside a stash slot
  int next_src = -1;            // the layer whose output the next compute layer reads (-1: stage input)
  // an open block of parallel branches
  bool in_block = false, branch_open = false, branch_first_pending = false;
  int blk_src = -1, blk_width = -1, blk_ch = 0, blk_hh = 1, blk_ww = 1, nbr = 0, coff = 0, blk_oh = 0, blk_ow = 0;
  int b_first[pd::kMaxBranches], b_last[pd::kMaxBranches], b_coff[pd::kMaxBranches], b_c[pd::kMaxBranches];
  auto close_branch = [&](int i) -> int {
    if ((int)p.lin.size() == 0 || b_first[nbr] > (int)p.lin.size() - 1)
      return fail(PD_EINVAL, "layer %d: a branch needs at least one layer", i);
    if (nbr > 0 && (hh != blk_oh || ww != blk_ow))
      return fail(PD_EINVAL, "layer %d: branch %d ends at %dx%d, the others at %dx%d", i, nbr, hh, ww, blk_oh, blk_ow);
    blk_oh = hh; blk_ow = ww;
    b_last[nbr] = (int)p.lin.size() - 1;
    b_coff[nbr] = coff; b_c[nbr] = ch;
    p.lin[b_last[nbr]].br_last = true;
    coff += ch;
    ++nbr;
    branch_open = false;
    return PD_OK;
  };
  for (int i = 0; i < c->n_layers; ++i) {
    const pd_layer_desc& d = c->layers[i];
    if (p.has_loss) return fail(PD_EINVAL, "PD_SOFTMAX_XENT must be the last layer");
    if (d.kind == PD_CONCAT_BEGIN || d.kind == PD_BRANCH || d.kind == PD_CONCAT_END) {
      if (!p.bf16) return fail(PD_EINVAL, "layer %d: branched blocks are only built for PD_BF16_F32ACC", i);
      if (d.kind == PD_CONCAT_BEGIN) {
        if (in_block) return fail(PD_EINVAL, "layer %d: blocks do not nest", i);
        if (rows != p.B) return fail(PD_EINVAL, "layer %d: a block cannot follow an LSTM", i);
        in_block = true; branch_open = false; nbr = 0; coff = 0;
        blk_src = next_src; blk_width = width; blk_ch = ch; blk_hh = hh; blk_ww = ww;
      } else if (d.kind == PD_BRANCH) {
        if (!in_block) return fail(PD_EINVAL, "layer %d: PD_BRANCH outside a block", i);
        if (branch_open) { const int rc = close_branch(i); if (rc) return rc; }
        if (nbr >= pd::kMaxBranches) return fail(PD_EINVAL, "layer %d: more than %d branches", i, pd::kMaxBranches);
        branch_open = true; branch_first_pending = true;
        b_first[nbr] = (int)p.lin.size();
        next_src = blk_src; width = blk_width; ch = blk_ch; hh = blk_hh; ww = blk_ww;
      } else {
        if (!in_block || !branch_open) return fail(PD_EINVAL, "layer %d: PD_CONCAT_END without an open branch", i);
        const int rc = close_branch(i); if (rc) return rc;
        Layer L;
        L.kind = K_CONCAT;
        L.ih = L.oh = blk_oh; L.iw = L.ow = blk_ow; L.ic = L.oc = coff;
        L.in = L.out = blk_oh * blk_ow * coff;
        L.rows = p.B; L.src = -1; L.nbr = nbr; L.blk_src = blk_src;
        const int me = (int)p.lin.size();
        size_t dyo = 0;
        for (int b = 0; b < nbr; ++b) {
          L.b_first[b] = b_first[b]; L.b_last[b] = b_last[b]; L.b_coff[b] = b_coff[b]; L.b_c[b] = b_c[b];
          for (int q = b_first[b]; q <= b_last[b]; ++q) p.lin[q].block = me;
          p.lin[b_last[b]].bdy_off = dyo;
          dyo += align_up((size_t)p.B * blk_oh * blk_ow * b_c[b] * 2, 256);
        }
        if (dyo > p.blk_dy_bytes) p.blk_dy_bytes = dyo;
        // stage input width is known only once a layer has stated it: take it from the branch's first layer
        L.blk_in_elems = (size_t)p.lin[b_first[0]].rows * p.lin[b_first[0]].in;
        const size_t stride = align_up(L.blk_in_elems * 2, 256);
        for (int b = 0; b < nbr; ++b) {
          if ((size_t)p.lin[b_first[b]].in != (size_t)p.lin[b_first[0]].in)
            return fail(PD_EINVAL, "layer %d: the branches disagree on the block's input size", i);
          p.lin[b_first[b]].bdx_off = (size_t)b * stride;
        }
        if (stride > p.blk_dx_stride) p.blk_dx_stride = stride;
        if (stride * nbr > p.blk_dx_bytes) p.blk_dx_bytes = stride * nbr;
        p.lin.push_back(L);
        in_block = false;
        width = L.out; ch = coff; hh = blk_oh; ww = blk_ow;
        next_src = me;
        Layer& C = p.lin.back();
        C.y_off = y_off; y_off = align_up(y_off + (size_t)C.rows * C.out * 4, 256);
        const size_t ab = align_up((size_t)C.rows * C.out * p.esz, 256);
        if (ab > p.pp_bytes) p.pp_bytes = ab;
      }
      continue;
    }
    if (in_block && !branch_open) return fail(PD_EINVAL, "layer %d: a layer inside a block must follow PD_BRANCH", i);
    if (in_block && d.kind != PD_CONV2D && d.kind != PD_MAXPOOL2D && d.kind != PD_AVGPOOL2D)
      return fail(PD_EINVAL, "layer %d: only convolution and pooling layers may sit inside a block", i);
    if (d.kind == PD_LINEAR) {
      Layer L;
      L.kind = K_LINEAR;
      L.in = d.p[0]; L.out = d.p[1]; L.relu = d.p[2] != 0;
      if (L.in < 1 || L.out < 1) return fail(PD_EINVAL, "layer %d: bad Linear shape %dx%d", i, L.out, L.in);
      if (width >= 0 && L.in != width) return fail(PD_EINVAL, "layer %d: in_features %d != previous width %d", i, L.in, width);
      if (p.bf16 && ((L.in % 8) || (L.out % 8)))
        return fail(PD_EINVAL, "layer %d: bf16 mode needs in/out features divisible by 8 (got %d, %d)", i, L.in, L.out);
      L.ic = L.in; L.oc = L.out;
      L.n_w = (size_t)L.in * L.out; L.n_b = L.out;
      width = L.out; ch = L.out; hh = ww = 1;
      L.rows = rows;
      L.dz_off = dz_off; dz_off = align_up(dz_off + (size_t)rows * L.out * p.esz, 256);
      p.lin.push_back(L);
    } else if (d.kind == PD_LSTM) {
      Layer L;
      L.kind = K_LSTM;
      L.in = d.p[0]; L.out = d.p[1]; L.T = d.p[2];
      if (!p.bf16) return fail(PD_EINVAL, "layer %d: the LSTM is only built for PD_BF16_F32ACC", i);
      if (L.in < 8 || L.out < 8 || (L.in % 8) || (L.out % 8) || L.T < 1)
        return fail(PD_EINVAL, "layer %d: LSTM needs input and hidden sizes divisible by 8 and seq_len >= 1", i);
      if (rows != p.B && rows != p.B * L.T) return fail(PD_EINVAL, "layer %d: sequence length differs from the layer below", i);
      if (width >= 0 && rows == p.B) return fail(PD_EINVAL, "layer %d: an LSTM must be first in its stage or follow an LSTM", i);
      if (width >= 0 && L.in != width) return fail(PD_EINVAL, "layer %d: LSTM input size %d != previous width %d", i, L.in, width);
      rows = p.B * L.T;
      L.rows = rows; L.ic = L.in; L.oc = L.out;
      L.n_w = (size_t)4 * L.out * L.in + (size_t)4 * L.out * L.out; L.n_b = (size_t)4 * L.out;
      width = L.out; ch = L.out; hh = ww = 1;
      L.dz_off = dz_off; dz_off = align_up(dz_off + (size_t)rows * 4 * L.out * 2, 256);
      L.dc_off = dz_off; dz_off = align_up(dz_off + (size_t)p.B * L.out * 4, 256);
      p.lin.push_back(L);
    } else if (d.kind == PD_CONV2D) {
      Layer L;
      L.kind = K_CONV;
      L.ic = d.p[0]; L.oc = d.p[1]; L.kh = d.p[2]; L.kw = d.p[3]; L.stride = d.p[4]; L.ph = d.p[5]; L.pw = d.p[6];
      L.relu = d.p[7] != 0; L.ih = d.p[8]; L.iw = d.p[9];
      if (!p.bf16) return fail(PD_EINVAL, "layer %d: convolution is only built for PD_BF16_F32ACC", i);
      if (L.ic < 1 || L.oc < 1 || L.kh < 1 || L.kw < 1 || L.stride < 1 || L.ph < 0 || L.pw < 0 || L.ih < 1 || L.iw < 1)
        return fail(PD_EINVAL, "layer %d: bad convolution geometry", i);
      L.oh = (L.ih + 2 * L.ph - L.kh) / L.stride + 1;
      L.ow = (L.iw + 2 * L.pw - L.kw) / L.stride + 1;
      if (L.oh < 1 || L.ow < 1) return fail(PD_EINVAL, "layer %d: empty convolution output", i);
      L.in = L.ih * L.iw * L.ic; L.out = L.oh * L.ow * L.oc;
      if (width >= 0 && (L.in != width || L.ic != ch || L.ih != hh || L.iw != ww))
        return fail(PD_EINVAL, "layer %d: convolution input %dx%dx%d does not match the previous output %dx%dx%d", i,
                    L.ih, L.iw, L.ic, hh, ww, ch);
      const bool smallk = L.kh * L.kw * L.ic <= 32 && L.oc <= 64;
      if (L.oc % 8 || (!smallk && L.ic % 8))
        return fail(PD_EINVAL, "layer %d: channel counts must be divisible by 8 (a first layer with kh*kw*Cin <= 32 and "
                    "Cout <= 64 is exempt on the input side); got %d -> %d", i, L.ic, L.oc);
      L.n_w = (size_t)L.oc * L.kh * L.kw * L.ic; L.n_b = L.oc;
      pd::ConvGeom g = {p.B, L.ih, L.iw, L.ic, L.oh, L.ow, L.oc, L.kh, L.kw, L.stride, L.ph, L.pw};
      L.splits = pd::conv_wgrad_split_count(g);
      L.part_off = part_off; part_off = align_up(part_off + (size_t)L.splits * (L.n_w + L.n_b) * 4, 256);
      if (L.n_w * 2 > p.wt_bytes) p.wt_bytes = align_up(L.n_w * 2, 256);
      width = L.out; ch = L.oc; hh = L.oh; ww = L.ow;
      p.lin.push_back(L);
    } else if (d.kind == PD_MAXPOOL2D || d.kind == PD_AVGPOOL2D) {
      Layer L;
      const bool is_max = d.kind == PD_MAXPOOL2D;
      L.kh = L.kw = d.p[0]; L.stride = d.p[1];
      L.ph = L.pw = is_max ? 0 : d.p[2];
      const int* q = is_max ? d.p + 2 : d.p + 3;
      L.ic = L.oc = q[0]; L.ih = q[1]; L.iw = q[2];
      L.is_max = is_max;
      if (!p.bf16) return fail(PD_EINVAL, "layer %d: pooling is only built for PD_BF16_F32ACC", i);
      if (L.kh < 1 || L.stride < 1 || L.ph < 0 || L.ph >= L.kh || L.ic < 8 || (L.ic % 8) || L.ih + 2 * L.ph < L.kh ||
          L.iw + 2 * L.pw < L.kh)
        return fail(PD_EINVAL, "layer %d: pooling needs window >= 1, stride >= 1, 0 <= pad < window <= padded input, "
                    "channels divisible by 8", i);
      L.kind = (is_max && L.kh == 2 && L.stride == 2 && !(L.ih % 2) && !(L.iw % 2)) ? K_POOL : K_GPOOL;
      L.oh = (L.ih + 2 * L.ph - L.kh) / L.stride + 1; L.ow = (L.iw + 2 * L.pw - L.kw) / L.stride + 1;
      L.in = L.ih * L.iw * L.ic; L.out = L.oh * L.ow * L.oc;
      if (width >= 0 && (L.in != width || L.ic != ch || L.ih != hh || L.iw != ww))
        return fail(PD_EINVAL, "layer %d: pooling input does not match the previous output", i);
      width = L.out; ch = L.oc; hh = L.oh; ww = L.ow;
      p.lin.push_back(L);
    } else if (d.kind == PD_SOFTMAX_XENT) {
      if (p.lin.empty() || i == 0 || c->layers[i - 1].kind != PD_LINEAR)
        return fail(PD_EINVAL, "PD_SOFTMAX_XENT must follow a PD_LINEAR");
      if (d.p[0] != width) return fail(PD_EINVAL, "loss classes %d != logits width %d", d.p[0], width);
      if (p.lin.back().relu) return fail(PD_EINVAL, "the Linear feeding the loss must not have a ReLU");
      p.has_loss = true;
      p.classes = width;
    } else {
      return fail(PD_EINVAL, "layer %d: unknown kind %d", i, d.kind);
    }
    if (d.kind != PD_SOFTMAX_XENT) {
      Layer& L = p.lin.back();
      L.src = next_src;
      next_src = (int)p.lin.size() - 1;
      if (in_block && branch_first_pending) { L.br_first = true; branch_first_pending = false; }
      if (L.n_w) {
        L.flat_w = flat; flat += L.n_w;
        L.flat_b = flat; flat += L.n_b;
        L.w_off = dev; dev = align_up(dev + L.n_w, 128);
        L.b_off = dev; dev = align_up(dev + L.n_b, 128);
      }
      if (!L.rows) L.rows = p.B;
      if (p.bf16 && L.rows >= kBigRows && (L.kind == K_LINEAR || L.kind == K_LSTM)) {
        const int n_out = L.kind == K_LSTM ? 4 * L.out : L.out;
        L.splits = pd::conv_wgrad_split_count(rows_as_pixels(L.rows, L.in, n_out));
        L.part_off = part_off; part_off = align_up(part_off + (size_t)L.splits * ((size_t)n_out * L.in + n_out) * 4, 256);
        if (L.kind == K_LSTM) {
          L.splits2 = pd::conv_wgrad_split_count(rows_as_pixels(L.rows, L.out, n_out));
          L.part2_off = part_off;
          part_off = align_up(part_off + (size_t)L.splits2 * ((size_t)n_out * L.out + n_out) * 4, 256);
        }
      }
      if (L.kind == K_LSTM && (size_t)4 * L.out * L.out * 2 > p.wt_bytes) p.wt_bytes = align_up((size_t)4 * L.out * L.out * 2, 256);
      if (L.kind == K_LSTM) {
        L.y_off = y_off; y_off = align_up(y_off + (size_t)(L.T + 1) * p.B * L.out * 2, 256);
        L.g_off = y_off; y_off = align_up(y_off + (size_t)L.rows * 4 * L.out * 4, 256);
        L.c_off = y_off; y_off = align_up(y_off + (size_t)(L.T + 1) * p.B * L.out * 4, 256);
      } else {
        L.y_off = y_off; y_off = align_up(y_off + (size_t)L.rows * L.out * 4, 256);  // room for fp32 (logits)
      }
      if (L.kind != K_LINEAR) {
        const size_t ab = align_up((size_t)L.rows * (L.in > L.out ? L.in : L.out) * p.esz, 256);
        if (ab > p.pp_bytes) p.pp_bytes = ab;
      }
      (void)x_off;
    }
  }
  if (in_block) return fail(PD_EINVAL, "a block is still open at the end of the layer list");
  if (p.lin.empty()) return fail(PD_EINVAL, "stage has no compute layer");
  p.part_bytes = part_off;
  p.n_params = flat;
  p.p_pad = dev;
  p.in_bytes = align_up((size_t)p.lin.front().rows * p.lin.front().in * p.esz, 256);
  p.out_bytes = align_up((size_t)p.lin.back().rows * p.lin.back().out * p.esz, 256);
  p.dlogits_off = y_off;
  if (p.has_loss) y_off = align_up(y_off + (size_t)p.lin.back().rows * p.classes * p.esz, 256);
  p.stash_slot_bytes = y_off;
  p.dz_bytes = dz_off;
  if (p.bf16)
    for (const Layer& L : p.lin) {
      if (L.kind != K_LINEAR && L.kind != K_LSTM) continue;
      size_t w = pd::gemm_bf16_workspace_bytes(L.rows, L.kind == K_LSTM ? 4 * L.out : L.out, L.in);
      if (L.kind == K_LSTM) {  // the per-step recurrent products always leave partial sums in the workspace
        size_t r = pd::gemm_bf16_workspace_bytes(p.B, 4 * L.out, L.out);
        const size_t r2 = pd::gemm_bf16_workspace_bytes(p.B, L.out, 4 * L.out);
        if (r2 > r) r = r2;
        const size_t one = (size_t)p.B * 4 * L.out * 4;
        if (r < one) r = one;
        if (r > w) w = r;
      }
      if (p.has_loss && &L == &p.lin.back()) {  // the logits may be left as partial sums for the loss kernel
        const size_t one = (size_t)L.rows * L.out * 4;
        if (one > w) w = one;
      }
      if (L.splits > 0) {  // many rows: room for the transposed operands of the weight-gradient products
        const int n_out = L.kind == K_LSTM ? 4 * L.out : L.out;
        const size_t t1 = pd::linear_wgrad_big_scratch_bytes(L.rows, n_out, L.in > L.out ? L.in : L.out);
        if (t1 > w) w = t1;
        const size_t t2 = pd::linear_wgrad_update_big_scratch_bytes(L.rows, n_out, L.in);  // split row sums
        if (t2 > w) w = t2;
        if (L.kind == K_LSTM) {
          const size_t t3 = pd::linear_wgrad_update_big_scratch_bytes(L.rows, n_out, L.out);
          if (t3 > w) w = t3;
        }
      }
      if (w > p.ws_bytes) p.ws_bytes = w;
    }
  p.ws_bytes = align_up(p.ws_bytes, 256);
  size_t o = 0;
  if (!secondary) {
    p.o_ring = o; o += align_up((size_t)p.ring_depth * p.p_pad * p.esz, 256);
    if (p.bf16) { p.o_master = o; o += align_up(p.p_pad * 4, 256); }
    if (p.bf16 && p.replicas <= 1) {
      for (Layer& L : p.lin)
        if (L.n_w && L.kind != K_CONV && L.splits == 0) { L.split_master = true; p.any_split = true; }
      if (p.any_split) { p.o_rem = o; o += align_up(p.p_pad * 2, 256); }
    }
    p.o_mom = o; o += align_up(p.p_pad * 4, 256);
  }
  if (p.replicas > 1) { p.o_gradbuf = o; o += align_up(p.p_pad * 4, 256); }
  p.o_in = o; o += (size_t)p.in_depth * p.in_bytes;
  p.o_stash = o; o += (size_t)p.depth * p.stash_slot_bytes;
  p.o_dz = o; o += p.dz_bytes * (p.lane_b ? 2 : 1);  // (two sets with a backward stream)
  if (!p.has_loss) { p.o_grad = o; o += 2 * p.out_bytes; }
  p.o_ws = o; o += p.ws_bytes;
  if (p.lane_b) { p.o_ws_b = o; o += p.ws_bytes; }
  p.o_pp = o; o += 2 * p.pp_bytes;
  p.o_part = o; o += p.part_bytes * (p.lane_b ? 2 : 1);
  p.o_wt = o; o += p.wt_bytes;
  p.o_blk_dy = o; o += p.blk_dy_bytes;
  p.o_blk_dx = o; o += p.blk_dx_bytes;
  p.o_rowloss = o; o += align_up((size_t)p.lin.back().rows * 4, 256);
  p.o_seq = o; o += align_up((size_t)2 * pd::kSeqSyncWords * sizeof(unsigned), 256);
  p.total = o;
  return PD_OK;
}


// ---- multi-step recurrence kernels: host side ------------------------------------------------------------------
// Such a kernel needs its whole grid resident at once and takes almost every compute unit's LDS.  Two of them
// dispatched together (two stages on two streams, or a stage's forward and backward lanes) could each get part of the
// chip and wait for the rest until their spin limits expire, so all launches of one process are chained: each waits
// for the event of the one before it, on whatever stream that was.
int g_seq_mode = 1;                     // 1: multi-step kernels where they apply (default); 0: one launch per time step
unsigned g_seq_spin_limit = 4000000u;   // polls (each at least a memory round trip) before a workgroup gives up
unsigned g_seq_starve = 0u;     // test hook: no workgroup publishes its results
struct SeqChain {
  std::mutex mu;
  std::map<int, std::vector<hipEvent_t>> ring;  // per device
  std::map<int, size_t> next;
  std::map<int, hipEvent_t> last;
};
SeqChain& seq_chain() { static SeqChain c; return c; }
constexpr size_t kSeqChainEvents = 64;

// call with the launch's stream BEFORE the launch (wait for the previous multi-step kernel) ...
hipError_t seq_chain_enter(hipStream_t s) {
  SeqChain& c = seq_chain();
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  std::lock_guard<std::mutex> g(c.mu);
  auto it = c.last.find(dev);
  if (it != c.last.end() && it->second) e = hipStreamWaitEvent(s, it->second, 0);
  return e;
}
// ... and AFTER it (this launch becomes the one to wait for)
hipError_t seq_chain_leave(hipStream_t s) {
  SeqChain& c = seq_chain();
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  std::lock_guard<std::mutex> g(c.mu);
  std::vector<hipEvent_t>& ring = c.ring[dev];
  if (ring.empty()) {
    ring.assign(kSeqChainEvents, nullptr);
    for (hipEvent_t& ev : ring) {
      e = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
      if (e != hipSuccess) { ring.clear(); return e; }
    }
  }
  hipEvent_t ev = ring[c.next[dev]++ % kSeqChainEvents];
  e = hipEventRecord(ev, s);
  if (e == hipSuccess) c.last[dev] = ev;
  return e;
}

// (Not under stream capture: the chain's events lie outside the capture, and a replayed graph would bypass the chain.)
// Where a max-pooling layer keeps the routing record of a minibatch (four bits per output element for the 2x2 kernel,
// a byte for the general one): behind its bf16 output in the layer's region of the stash slot, which is laid out for
// four bytes per element.  (Always the
// slot's own region, also when the stage's last output lives in a buffer borrowed from the consumer.)
static uint32_t* pool_route(const pd_stage* st, char* slot, const Linear& L) {
  return reinterpret_cast<uint32_t*>(slot + L.y_off + (size_t)L.rows * L.out * 2);
}

bool seq_wanted(const pd_stage* st, hipStream_t s, int B, int H, int T) {
  if (g_seq_mode != 1 || !st->bf16 || !st->seq_sync || !pd::lstm_seq_applies(B, H, T, st->n_cus)) return false;
  hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
  return hipStreamIsCapturing(s, &cs) == hipSuccess && cs == hipStreamCaptureStatusNone;
}

// After a synchronisation: has a multi-step kernel of this stage given up waiting for its peers?
int seq_check(pd_stage* st) {
  if (!st->seq_used) return PD_OK;
  st->seq_used = false;
  unsigned flags[2] = {0u, 0u};
  for (int d = 0; d < 2; ++d)
    PD_HIP(hipMemcpy(&flags[d], st->seq_sync + d * pd::kSeqSyncWords + pd::kSeqStatusWord, sizeof(unsigned), hipMemcpyDeviceToHost));
  if (!flags[0] && !flags[1]) return PD_OK;
  PD_HIP(hipMemset(st->seq_sync, 0, (size_t)2 * pd::kSeqSyncWords * sizeof(unsigned)));
  return fail(PD_ESTATE, "a multi-step recurrence kernel gave up waiting for its peer workgroups (%s pass): the stage's "
              "activations, gradients and weights after that minibatch are not valid", flags[0] ? "forward" : "backward");
}

int check_stage(const pd_stage* st) { return st ? PD_OK : fail(PD_EINVAL, "stage is null"); }

// The parameter state of a replicated stage lives with its primary: calls that write it go there.
int check_owner(const pd_stage* st) {
  if (check_stage(st)) return PD_EINVAL;
  return st->primary ? fail(PD_ESTATE, "this is a secondary replica: the parameter state belongs to its primary") : PD_OK;
}

// primary == null: an ordinary stage (or the primary of a replicated one); otherwise a further replica of it
int create_stage(const pd_stage_config* cfg, pd_stage* primary, void* stream, void* device_arena, size_t arena_bytes,
                 pd_stage** out) {
  if (!out) return fail(PD_EINVAL, "out is null");
  *out = nullptr;
  Plan p;
  const int rc = make_plan(cfg, p, primary != nullptr);
  if (rc != PD_OK) return rc;
  if (!device_arena) return fail(PD_EINVAL, "device_arena is null");
  if (reinterpret_cast<uintptr_t>(device_arena) & 255u) return fail(PD_EINVAL, "device_arena must be 256-byte aligned");
  if (arena_bytes < p.total) return fail(PD_ENOMEM, "arena has %zu bytes, stage needs %zu", arena_bytes, p.total);
  pd_stage* st = new (std::nothrow) pd_stage();
  if (!st) return fail(PD_ENOMEM, "host allocation failed");
  char* a = static_cast<char*>(device_arena);
  st->cfg = *cfg;
  st->cfg_layers.assign(cfg->layers, cfg->layers + cfg->n_layers);
  st->cfg.layers = st->cfg_layers.data();
  st->stage_index = cfg->stage_index; st->num_stages = cfg->num_stages; st->noam = cfg->noam;
  st->depth = p.depth; st->in_depth = p.in_depth; st->ring_depth = p.ring_depth; st->vsync = cfg->vertical_sync != 0;
  st->B = p.B; st->bf16 = p.bf16; st->has_loss = p.has_loss;
  st->classes = p.classes;
  st->rule = pd::UpdateRule{cfg->lr, cfg->momentum, cfg->eps, cfg->optimizer};
  st->stream = static_cast<hipStream_t>(stream);
  st->cfg.stream = stream;
  st->lin = p.lin; st->esz = p.esz; st->n_params = p.n_params; st->p_pad = p.p_pad;
  st->in_bytes = p.in_bytes; st->out_bytes = p.out_bytes; st->stash_slot_bytes = p.stash_slot_bytes;
  st->dlogits_off = p.dlogits_off;
  st->n_replicas = p.replicas;
  if (primary) {
    st->primary = primary;
    st->ring = primary->ring; st->master = primary->master; st->mom = primary->mom;
    st->latest = primary->latest;
  } else {
    st->ring = a + p.o_ring;
    st->master = p.bf16 ? reinterpret_cast<float*>(a + p.o_master) : nullptr;
    st->rem = p.any_split ? reinterpret_cast<uint16_t*>(a + p.o_rem) : nullptr;
    st->mom = reinterpret_cast<float*>(a + p.o_mom);
  }
  st->gradbuf = p.replicas > 1 ? reinterpret_cast<float*>(a + p.o_gradbuf) : nullptr;
  st->in_ring = a + p.o_in; st->stash = a + p.o_stash; st->dz = a + p.o_dz;
  st->grad_in = p.has_loss ? nullptr : a + p.o_grad;
  st->ws = reinterpret_cast<float*>(a + p.o_ws); st->ws_bytes = p.ws_bytes;
  if (p.lane_b && !primary) {
    st->stream_b = static_cast<hipStream_t>(cfg->stream_backward);
    st->ws_b = reinterpret_cast<float*>(a + p.o_ws_b);
  }
  st->row_loss = reinterpret_cast<float*>(a + p.o_rowloss);
  st->seq_sync = reinterpret_cast<unsigned*>(a + p.o_seq);
  {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess) st->n_cus = n;
  }
  st->pp = a + p.o_pp; st->pp_bytes = p.pp_bytes; st->part = a + p.o_part; st->wt = a + p.o_wt;
  st->dz_base = st->dz; st->part_base = st->part;
  st->dz_set_bytes = p.dz_bytes; st->part_set_bytes = p.part_bytes;
  st->blk_dy = a + p.o_blk_dy; st->blk_dx = a + p.o_blk_dx; st->blk_dx_stride = p.blk_dx_stride;
  st->borrowed_out.assign(p.depth, nullptr);
  hipError_t e = primary ? hipSuccess : pd::fill_zero(st->stream, st->mom, p.p_pad * 4);
  if (e == hipSuccess) e = pd::fill_zero(st->stream, st->seq_sync, (size_t)2 * pd::kSeqSyncWords * sizeof(unsigned));
  // padding between layers inside the gradient buffer is never written by a gradient kernel: keep it at zero
  if (e == hipSuccess && st->gradbuf) e = pd::fill_zero(st->stream, st->gradbuf, p.p_pad * 4);
  if (e == hipSuccess && st->gradbuf) e = hipEventCreateWithFlags(&st->ev_rep, hipEventDisableTiming);
  for (hipEvent_t* ev : {&st->ev_upd[0], &st->ev_upd[1], &st->ev_bwd})
    if (e == hipSuccess && st->stream_b) e = hipEventCreateWithFlags(ev, hipEventDisableTiming);
  if (st->stream_b) st->ev_fwd.assign(st->depth, nullptr);
  for (hipEvent_t& ev : st->ev_fwd)
    if (e == hipSuccess) e = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
  for (int d = 0; d < st->depth && e == hipSuccess; ++d)
    for (const Linear& L : st->lin)
      if (L.kind == K_LSTM && e == hipSuccess) {
        char* slot = st->stash + (size_t)d * st->stash_slot_bytes;
        e = pd::fill_zero(st->stream, slot + L.y_off, (size_t)st->B * L.out * 2);
        if (e == hipSuccess) e = pd::fill_zero(st->stream, slot + L.c_off, (size_t)st->B * L.out * 4);
      }
  if (e != hipSuccess) {
    for (hipEvent_t ev : {st->ev_rep, st->ev_upd[0], st->ev_upd[1], st->ev_bwd})
      if (ev) (void)hipEventDestroy(ev);
    for (hipEvent_t ev : st->ev_fwd)
      if (ev) (void)hipEventDestroy(ev);
    delete st;
    return fail(PD_EHIP, "clearing momentum and initial states: %s", hipGetErrorString(e));
  }
  if (primary) primary->secondaries.push_back(st);
  *out = st;
  return PD_OK;
}

}  // namespace

extern "C" {

const char* pd_last_error(void) { return g_err.c_str(); }

int pd_schedule_1f1b(int32_t num_stages, int32_t noam, int32_t num_minibatches, int32_t stage_index, pd_op* out,
                     size_t cap, size_t* n_out) {
  if (num_stages < 1 || stage_index < 0 || stage_index >= num_stages || noam < 1 || num_minibatches < 0)
    return fail(PD_EINVAL, "bad schedule arguments (S=%d noam=%d M=%d s=%d)", num_stages, noam, num_minibatches, stage_index);
  return emit_schedule(stage_depth(num_stages, noam, stage_index), num_minibatches, out, cap, n_out);
}

int pd_schedule_1f1b_vertical_sync(int32_t num_stages, int32_t noam, int32_t num_minibatches, int32_t stage_index,
                                   pd_op* out, size_t cap, size_t* n_out) {
  if (num_stages < 1 || noam < 1 || num_minibatches < 0 || stage_index < 0 || stage_index >= num_stages)
    return fail(PD_EINVAL, "bad schedule arguments (S=%d noam=%d M=%d s=%d)", num_stages, noam, num_minibatches, stage_index);
  // same op order as the stage's own list; F and B carry the version the INPUT stage's forward read
  std::vector<pd_op> own, first;
  const int ring = stage_depth(num_stages, noam, 0);
  build_schedule(stage_depth(num_stages, noam, stage_index), num_minibatches, own);
  build_schedule(ring, num_minibatches, first);
  std::vector<int> tag(num_minibatches > 0 ? num_minibatches : 0, 0);
  for (const pd_op& o : first)
    if (o.kind == PD_OP_F) tag[o.mb_id] = o.version;
  for (pd_op& o : own) {
    if (o.kind != PD_OP_U) o.version = tag[o.mb_id];
    o.slot = o.version % ring;
  }
  if (n_out) *n_out = own.size();
  if (own.size() > cap) return fail(PD_ENOMEM, "schedule needs %zu entries, capacity %zu", own.size(), cap);
  if (!own.empty()) {
    if (!out) return fail(PD_EINVAL, "out is null");
    memcpy(out, own.data(), own.size() * sizeof(pd_op));
  }
  return PD_OK;
}

int pd_schedule_1f1b_depth(int32_t depth, int32_t num_minibatches, pd_op* out, size_t cap, size_t* n_out) {
  if (depth < 1 || num_minibatches < 0) return fail(PD_EINVAL, "bad schedule arguments (depth=%d M=%d)", depth, num_minibatches);
  return emit_schedule(depth, num_minibatches, out, cap, n_out);
}

int pd_stage_query_bytes(const pd_stage_config* cfg, size_t* device_bytes) {
  if (!device_bytes) return fail(PD_EINVAL, "device_bytes is null");
  Plan p;
  const int rc = make_plan(cfg, p);
  if (rc != PD_OK) return rc;
  *device_bytes = p.total;
  return PD_OK;
}

int pd_stage_create(const pd_stage_config* cfg, void* device_arena, size_t arena_bytes, pd_stage** out) {
  if (!cfg) return fail(PD_EINVAL, "config is null");
  return create_stage(cfg, nullptr, cfg->stream, device_arena, arena_bytes, out);
}

int pd_replica_route(int32_t mb_id, int32_t n_replicas, int32_t* replica, int32_t* round) {
  if (mb_id < 0 || n_replicas < 1) return fail(PD_EINVAL, "bad routing arguments (minibatch %d, %d replicas)", mb_id, n_replicas);
  if (replica) *replica = mb_id % n_replicas;
  if (round) *round = mb_id / n_replicas;
  return PD_OK;
}

int pd_stage_replica_query_bytes(const pd_stage_config* cfg, size_t* device_bytes) {
  if (!device_bytes) return fail(PD_EINVAL, "device_bytes is null");
  Plan p;
  const int rc = make_plan(cfg, p, true);
  if (rc != PD_OK) return rc;
  *device_bytes = p.total;
  return PD_OK;
}

int pd_stage_create_replica(pd_stage* primary, void* stream, void* device_arena, size_t arena_bytes, pd_stage** out) {
  if (out) *out = nullptr;
  if (check_stage(primary)) return PD_EINVAL;
  if (primary->primary) return fail(PD_EINVAL, "replicas are created from the primary");
  if (primary->n_replicas < 2) return fail(PD_EINVAL, "the stage is not configured as replicated");
  if ((int)primary->secondaries.size() + 1 >= primary->n_replicas)
    return fail(PD_ESTATE, "the stage already has its %d replicas", primary->n_replicas);
  if (!primary->in_flight.empty() || primary->grad_pending) return fail(PD_ESTATE, "minibatches in flight");
  return create_stage(&primary->cfg, primary, stream, device_arena, arena_bytes, out);
}

int pd_stage_destroy(pd_stage* st) {
  if (!st) return PD_OK;
  if (!st->secondaries.empty()) return fail(PD_ESTATE, "destroy the %zu further replicas of this stage first", st->secondaries.size());
  if (st->primary) {
    auto& v = st->primary->secondaries;
    v.erase(std::remove(v.begin(), v.end(), st), v.end());
  }
  for (hipEvent_t ev : {st->ev_rep, st->ev_upd[0], st->ev_upd[1], st->ev_bwd})
    if (ev) (void)hipEventDestroy(ev);
  for (auto* v : {&st->ev_f, &st->ev_b, &st->ev_u, &st->mark_pool, &st->ev_fwd})
    for (hipEvent_t e : *v) (void)hipEventDestroy(e);
  for (const pd_stage::Mark& m : st->marks) (void)hipEventDestroy(m.ev);
  delete st;
  return PD_OK;
}

int pd_stage_num_params(const pd_stage* st, size_t* n) {
  if (check_stage(st) || !n) return fail(PD_EINVAL, "null argument");
  *n = st->n_params;
  return PD_OK;
}

int pd_stage_depth(const pd_stage* st, int32_t* depth, int32_t* input_ring_depth) {
  if (check_stage(st)) return PD_EINVAL;
  if (depth) *depth = st->depth;
  if (input_ring_depth) *input_ring_depth = st->in_depth;
  return PD_OK;
}

int pd_stage_ring_depth(const pd_stage* st, int32_t* ring_depth) {
  if (check_stage(st) || !ring_depth) return fail(PD_EINVAL, "null argument");
  *ring_depth = st->ring_depth;
  return PD_OK;
}

// Layers whose master weights live as ring copy + remainder: fp32 values in the staging area -> version `version`'s
// ring slot and the remainders / the other way round (always from the latest version).  Enqueued on the stage's
// stream.
static hipError_t split_master_from_staging(pd_stage* st, int version) {
  pd::bf16_t* r = reinterpret_cast<pd::bf16_t*>(st->ring_slot(version));
  for (const Linear& L : st->lin)
    if (L.split_master) {
      hipError_t e = pd::master_split(st->stream, st->master + L.w_off, r + L.w_off, st->rem + L.w_off, L.n_w);
      if (e != hipSuccess) return e;
    }
  return hipSuccess;
}
static hipError_t materialize_master(pd_stage* st) {
  const pd::bf16_t* r = reinterpret_cast<const pd::bf16_t*>(st->ring_slot(st->latest));
  for (const Linear& L : st->lin)
    if (L.split_master) {
      hipError_t e = pd::master_merge(st->stream, r + L.w_off, st->rem + L.w_off, st->master + L.w_off, L.n_w);
      if (e != hipSuccess) return e;
    }
  return hipSuccess;
}

int pd_stage_set_params(pd_stage* st, const float* host_params, size_t n) {
  if (check_stage(st) || !host_params) return fail(PD_EINVAL, "null argument");
  if (check_owner(st)) return PD_ESTATE;
  if (n != st->n_params) return fail(PD_EINVAL, "expected %zu parameters, got %zu", st->n_params, n);
  PD_HIP(st->sync_all());
  if (const int seq_rc = seq_check(st)) return seq_rc;
  for (pd_stage* r : st->secondaries) {  // they read the same weights and restart with them
    PD_HIP(r->sync_all());
    r->latest = 0; r->last_fwd = -1; r->in_flight.clear(); r->grad_pending = false; r->trace.clear();
  }
  float* dst32 = st->bf16 ? st->master : reinterpret_cast<float*>(st->ring);
  for (const Linear& L : st->lin) {
    if (!L.n_w) continue;
    PD_HIP(hipMemcpy(dst32 + L.w_off, host_params + L.flat_w, L.n_w * 4, hipMemcpyHostToDevice));
    PD_HIP(hipMemcpy(dst32 + L.b_off, host_params + L.flat_b, L.n_b * 4, hipMemcpyHostToDevice));
    if (st->bf16) {
      pd::bf16_t* r = reinterpret_cast<pd::bf16_t*>(st->ring);
      if (!L.split_master) PD_HIP(pd::f32_to_bf16(st->stream, st->master + L.w_off, r + L.w_off, L.n_w));
      PD_HIP(pd::f32_to_bf16(st->stream, st->master + L.b_off, r + L.b_off, L.n_b));
    }
  }
  if (st->rem) PD_HIP(split_master_from_staging(st, 0));  // ring slot 0 = version 0
  PD_HIP(pd::fill_zero(st->stream, st->mom, st->p_pad * 4));
  PD_HIP(st->sync_all());
  if (const int seq_rc = seq_check(st)) return seq_rc;
  st->latest = 0; st->last_fwd = -1; st->in_flight.clear(); st->grad_pending = false; st->trace.clear();
  return PD_OK;
}

int pd_stage_get_params(pd_stage* st, int32_t version, int32_t ring_copy, float* host_out, size_t n) {
  if (check_stage(st) || !host_out) return fail(PD_EINVAL, "null argument");
  if (n != st->n_params) return fail(PD_EINVAL, "expected %zu parameters, got %zu", st->n_params, n);
  if (version < 0) version = st->latest;
  if (version > st->latest || version <= st->latest - st->ring_depth)
    return fail(PD_ESTATE, "version %d is not in the ring (latest %d, depth %d)", version, st->latest, st->ring_depth);
  PD_HIP(st->sync_all());
  if (const int seq_rc = seq_check(st)) return seq_rc;
  const bool from_master = st->bf16 && version == st->latest && !ring_copy;
  if (from_master && st->rem) {
    PD_HIP(materialize_master(st));
    PD_HIP(st->sync_all());
  if (const int seq_rc = seq_check(st)) return seq_rc;
  }
  if (!st->bf16 || from_master) {
    const float* src = from_master ? st->master : reinterpret_cast<const float*>(st->ring_slot(version));
    for (const Linear& L : st->lin) {
      if (!L.n_w) continue;
      PD_HIP(hipMemcpy(host_out + L.flat_w, src + L.w_off, L.n_w * 4, hipMemcpyDeviceToHost));
      PD_HIP(hipMemcpy(host_out + L.flat_b, src + L.b_off, L.n_b * 4, hipMemcpyDeviceToHost));
    }
    return PD_OK;
  }
  const uint16_t* src = reinterpret_cast<const uint16_t*>(st->ring_slot(version));
  std::vector<uint16_t> tmp;
  auto widen = [&](size_t dev_off, size_t flat_off, size_t cnt) -> hipError_t {
    tmp.resize(cnt);
    hipError_t e = hipMemcpy(tmp.data(), src + dev_off, cnt * 2, hipMemcpyDeviceToHost);
    if (e != hipSuccess) return e;
    for (size_t i = 0; i < cnt; ++i) {
      const uint32_t u = (uint32_t)tmp[i] << 16;
      memcpy(host_out + flat_off + i, &u, 4);
    }
    return hipSuccess;
  };
  for (const Linear& L : st->lin) {
    if (!L.n_w) continue;
    PD_HIP(widen(L.w_off, L.flat_w, L.n_w));
    PD_HIP(widen(L.b_off, L.flat_b, L.n_b));
  }
  return PD_OK;
}

int pd_stage_set_lr(pd_stage* st, float lr) {
  if (check_stage(st)) return PD_EINVAL;
  if (check_owner(st)) return PD_ESTATE;
  if (!(lr >= 0.f) || !std::isfinite(lr)) return fail(PD_EINVAL, "learning rate must be finite and >= 0");
  st->rule.lr = lr;  // read by the next update's launch; updates already enqueued keep the value they were launched with
  st->cfg.lr = lr;
  for (pd_stage* r : st->secondaries) { r->rule.lr = lr; r->cfg.lr = lr; }
  return PD_OK;
}

int pd_stage_set_momentum(pd_stage* st, const float* host_mom, size_t n) {
  if (check_stage(st) || !host_mom) return fail(PD_EINVAL, "null argument");
  if (check_owner(st)) return PD_ESTATE;
  if (n != st->n_params) return fail(PD_EINVAL, "expected %zu values, got %zu", st->n_params, n);
  if (!st->in_flight.empty() || st->grad_pending) return fail(PD_ESTATE, "minibatches in flight");
  PD_HIP(st->sync_all());
  if (const int seq_rc = seq_check(st)) return seq_rc;
  for (const Linear& L : st->lin) {
    if (!L.n_w) continue;
    PD_HIP(hipMemcpy(st->mom + L.w_off, host_mom + L.flat_w, L.n_w * 4, hipMemcpyHostToDevice));
    PD_HIP(hipMemcpy(st->mom + L.b_off, host_mom + L.flat_b, L.n_b * 4, hipMemcpyHostToDevice));
  }
  return PD_OK;
}

int pd_stage_get_momentum(pd_stage* st, float* host_out, size_t n) {
  if (check_stage(st) || !host_out) return fail(PD_EINVAL, "null argument");
  if (n != st->n_params) return fail(PD_EINVAL, "expected %zu values, got %zu", st->n_params, n);
  PD_HIP(st->sync_all());
  if (const int seq_rc = seq_check(st)) return seq_rc;
  for (const Linear& L : st->lin) {
    if (!L.n_w) continue;
    PD_HIP(hipMemcpy(host_out + L.flat_w, st->mom + L.w_off, L.n_w * 4, hipMemcpyDeviceToHost));
    PD_HIP(hipMemcpy(host_out + L.flat_b, st->mom + L.b_off, L.n_b * 4, hipMemcpyDeviceToHost));
  }
  return PD_OK;
}

// ---- per-stage checkpoint (Section 4, "Checkpointing") ----------------------------------------------------
// File: 8 bytes "PDCKPT1\0"; u32 precision; u32 0; u64 n_params; i64 latest version; u64 checksum; then n_params
// floats of the fp32 (master) weights and n_params floats of momentum, flat layout, little-endian.  The checksum
// runs over the two arrays, 8 bytes at a time: h = (h ^ word) * 0x100000001b3 starting from 0xcbf29ce484222325.
namespace {
constexpr char kCkptMagic[8] = {'P', 'D', 'C', 'K', 'P', 'T', '1', '\0'};
struct CkptHeader {
  char magic[8];
  uint32_t precision, zero;
  uint64_t n_params;
  int64_t latest;
  uint64_t checksum;
};
uint64_t ckpt_hash(uint64_t h, const float* p, size_t n) {  // n even or odd: the odd tail is widened with zero
  const size_t pairs = n / 2;
  for (size_t i = 0; i < pairs; ++i) {
    uint64_t w;
    memcpy(&w, p + 2 * i, 8);
    h = (h ^ w) * 0x100000001b3ull;
  }
  if (n & 1) {
    uint32_t t;
    memcpy(&t, p + n - 1, 4);
    h = (h ^ (uint64_t)t) * 0x100000001b3ull;
  }
  return h;
}
int ckpt_read(const char* path, CkptHeader& hd, std::vector<float>* w, std::vector<float>* m) {
  if (!path) return fail(PD_EINVAL, "checkpoint: path is null");
  FILE* f = fopen(path, "rb");
  if (!f) return fail(PD_EINVAL, "checkpoint: cannot open %s", path);
  int rc = PD_OK;
  std::vector<float> bw, bm;
  if (fread(&hd, sizeof hd, 1, f) != 1 || memcmp(hd.magic, kCkptMagic, 8) != 0 || hd.zero != 0 || hd.precision > 1 ||
      hd.latest < 0 || hd.latest > 0x7fffffff || hd.n_params > ((uint64_t)1 << 40)) {
    rc = fail(PD_EINVAL, "checkpoint: %s has no valid header", path);
  } else {
    bw.resize(hd.n_params);
    bm.resize(hd.n_params);
    char extra;
    if (fread(bw.data(), 4, bw.size(), f) != bw.size() || fread(bm.data(), 4, bm.size(), f) != bm.size() ||
        fread(&extra, 1, 1, f) != 0)
      rc = fail(PD_EINVAL, "checkpoint: %s is truncated or has trailing bytes", path);
    else if (ckpt_hash(ckpt_hash(0xcbf29ce484222325ull, bw.data(), bw.size()), bm.data(), bm.size()) != hd.checksum)
      rc = fail(PD_EINVAL, "checkpoint: %s fails its checksum", path);
  }
  fclose(f);
  if (rc == PD_OK && w) w->swap(bw);
  if (rc == PD_OK && m) m->swap(bm);
  return rc;
}
}  // namespace

int pd_checkpoint_info(const char* path, size_t* n_params, int32_t* latest, int32_t* precision) {
  CkptHeader hd;
  const int rc = ckpt_read(path, hd, nullptr, nullptr);
  if (rc != PD_OK) return rc;
  if (n_params) *n_params = (size_t)hd.n_params;
  if (latest) *latest = (int32_t)hd.latest;
  if (precision) *precision = (int32_t)hd.precision;
  return PD_OK;
}

int pd_stage_checkpoint_save(pd_stage* st, const char* path) {
  if (check_stage(st)) return PD_EINVAL;
  if (!path) return fail(PD_EINVAL, "checkpoint: path is null");
  if (st->grad_pending) return fail(PD_ESTATE, "checkpoint: a gradient is pending (save after pd_update)");
  std::vector<float> w(st->n_params), m(st->n_params);
  int rc = pd_stage_get_params(st, -1, 0, w.data(), w.size());
  if (rc == PD_OK) rc = pd_stage_get_momentum(st, m.data(), m.size());
  if (rc != PD_OK) return rc;
  CkptHeader hd;
  memcpy(hd.magic, kCkptMagic, 8);
  hd.precision = st->bf16 ? 1u : 0u;
  hd.zero = 0;
  hd.n_params = st->n_params;
  hd.latest = st->latest;
  hd.checksum = ckpt_hash(ckpt_hash(0xcbf29ce484222325ull, w.data(), w.size()), m.data(), m.size());
  FILE* f = fopen(path, "wb");
  if (!f) return fail(PD_EINVAL, "checkpoint: cannot create %s", path);
  const bool ok = fwrite(&hd, sizeof hd, 1, f) == 1 && fwrite(w.data(), 4, w.size(), f) == w.size() &&
                  fwrite(m.data(), 4, m.size(), f) == m.size();
  if (fclose(f) != 0 || !ok) return fail(PD_EINVAL, "checkpoint: writing %s failed", path);
  return PD_OK;
}

int pd_stage_checkpoint_load(pd_stage* st, const char* path) {
  if (check_stage(st)) return PD_EINVAL;
  CkptHeader hd;
  std::vector<float> w, m;
  int rc = ckpt_read(path, hd, &w, &m);
  if (rc != PD_OK) return rc;
  if (hd.n_params != st->n_params) return fail(PD_EINVAL, "checkpoint: %llu parameters, the stage has %zu", (unsigned long long)hd.n_params, st->n_params);
  if ((hd.precision == 1) != st->bf16) return fail(PD_EINVAL, "checkpoint: precision differs from the stage's");
  rc = pd_stage_set_params(st, w.data(), w.size());  // version 0 in ring slot 0, nothing in flight
  if (rc == PD_OK) rc = pd_stage_set_momentum(st, m.data(), m.size());
  if (rc != PD_OK) return rc;
  const int v = (int)hd.latest;
  if (v % st->ring_depth != 0)  // the weights belong in the ring slot of their version
    PD_HIP(hipMemcpy(st->ring_slot(v), st->ring_slot(0), st->p_pad * st->esz, hipMemcpyDeviceToDevice));
  st->latest = v;
  for (pd_stage* r : st->secondaries) r->latest = v;
  return PD_OK;
}

int pd_stage_overwrite_latest(pd_stage* st, const float* host_params, const float* host_mom, size_t n) {
  if (check_stage(st)) return PD_EINVAL;
  if (check_owner(st)) return PD_ESTATE;
  for (pd_stage* r : st->secondaries) {
    if (r->grad_pending) return fail(PD_ESTATE, "a gradient is pending on a replica: call pd_update_replicated first");
    PD_HIP(r->sync_all());
  }
  if (n != st->n_params) return fail(PD_EINVAL, "expected %zu values, got %zu", st->n_params, n);
  if (st->grad_pending) return fail(PD_ESTATE, "a gradient is pending: call pd_update first");
  PD_HIP(st->sync_all());
  if (const int seq_rc = seq_check(st)) return seq_rc;
  char* slot = st->ring_slot(st->latest);
  float* dst32 = st->bf16 ? st->master : reinterpret_cast<float*>(slot);
  for (const Linear& L : st->lin) {
    if (!L.n_w) continue;
    if (host_params) {
      PD_HIP(hipMemcpy(dst32 + L.w_off, host_params + L.flat_w, L.n_w * 4, hipMemcpyHostToDevice));
      PD_HIP(hipMemcpy(dst32 + L.b_off, host_params + L.flat_b, L.n_b * 4, hipMemcpyHostToDevice));
      if (st->bf16) {
        pd::bf16_t* r = reinterpret_cast<pd::bf16_t*>(slot);
        if (!L.split_master) PD_HIP(pd::f32_to_bf16(st->stream, st->master + L.w_off, r + L.w_off, L.n_w));
        PD_HIP(pd::f32_to_bf16(st->stream, st->master + L.b_off, r + L.b_off, L.n_b));
      }
    }
    if (host_mom) {
      PD_HIP(hipMemcpy(st->mom + L.w_off, host_mom + L.flat_w, L.n_w * 4, hipMemcpyHostToDevice));
      PD_HIP(hipMemcpy(st->mom + L.b_off, host_mom + L.flat_b, L.n_b * 4, hipMemcpyHostToDevice));
    }
  }
  if (host_params && st->rem) PD_HIP(split_master_from_staging(st, st->latest));
  PD_HIP(st->sync_all());
  if (const int seq_rc = seq_check(st)) return seq_rc;
  return PD_OK;
}

int pd_stage_check(pd_stage* st) {
  if (check_stage(st)) return PD_EINVAL;
  PD_HIP(st->sync_all());
  return seq_check(st);
}

int pd_stage_version(const pd_stage* st, int32_t mb_id, int32_t* version) {
  if (check_stage(st) || !version) return fail(PD_EINVAL, "null argument");
  if (mb_id < 0) {
    *version = st->latest;
    return PD_OK;
  }
  for (const InFlight& f : st->in_flight)
    if (f.mb == mb_id) {
      *version = f.version;
      return PD_OK;
    }
  return fail(PD_ESTATE, "minibatch %d is not in flight", mb_id);
}

int pd_stage_trace(const pd_stage* st, pd_op* out, size_t cap, size_t* n_out) {
  if (check_stage(st)) return PD_EINVAL;
  if (n_out) *n_out = st->trace.size();
  if (st->trace.size() > cap) return fail(PD_ENOMEM, "trace has %zu entries, capacity %zu", st->trace.size(), cap);
  if (!st->trace.empty()) {
    if (!out) return fail(PD_EINVAL, "out is null");
    std::copy(st->trace.begin(), st->trace.end(), out);
  }
  return PD_OK;
}

int pd_stage_set_trace_limit(pd_stage* st, size_t max_ops) {
  if (check_stage(st)) return PD_EINVAL;
  st->trace_cap = max_ops;
  while (st->trace.size() > max_ops) st->trace.pop_front();
  return PD_OK;
}

int pd_stage_input_slot(pd_stage* st, int32_t mb_id, void** dev_ptr) {
  if (check_stage(st) || !dev_ptr || mb_id < 0) return fail(PD_EINVAL, "bad argument");
  *dev_ptr = st->in_slot(mb_id);
  return PD_OK;
}

int pd_stage_grad_slot(pd_stage* st, int32_t mb_id, void** dev_ptr) {
  if (check_stage(st) || !dev_ptr || mb_id < 0) return fail(PD_EINVAL, "bad argument");
  if (st->has_loss) return fail(PD_ESTATE, "a stage that ends in the loss takes no output gradient");
  *dev_ptr = st->grad_slot(mb_id);
  return PD_OK;
}

int pd_stage_debug_read(pd_stage* st, int32_t what, int32_t mb_id, int32_t layer, float* host_out, size_t n) {
  if (check_stage(st) || !host_out || mb_id < 0) return fail(PD_EINVAL, "bad argument");
  const int nl = (int)st->lin.size();
  const char* src = nullptr;
  size_t cnt = 0;
  switch (what) {
    case 0:
      if (layer < 0 || layer >= nl) return fail(PD_EINVAL, "layer %d out of range", layer);
      src = st->out_of(st->stash_slot(mb_id), layer);
      cnt = (size_t)st->lin[layer].rows * st->lin[layer].out;
      break;
    case 1:
      src = st->in_slot(mb_id);
      cnt = (size_t)st->lin.front().rows * st->lin.front().in;
      break;
    case 2:
      if (st->has_loss) return fail(PD_ESTATE, "a stage that ends in the loss has no output-gradient slot");
      src = st->grad_slot(mb_id);
      cnt = (size_t)st->lin.back().rows * st->lin.back().out;
      break;
    case 3:
      if (layer < 0 || layer >= nl) return fail(PD_EINVAL, "layer %d out of range", layer);
      if (st->lin[layer].kind != K_LINEAR) return fail(PD_ESTATE, "layer %d does not keep its output gradient", layer);
      src = (st->has_loss && layer == nl - 1) ? st->stash_slot(mb_id) + st->dlogits_off : st->dz + st->lin[layer].dz_off;
      cnt = (size_t)st->lin[layer].rows * st->lin[layer].out;
      break;
    case 4:
      if (!st->has_loss) return fail(PD_ESTATE, "stage has no loss");
      src = st->stash_slot(mb_id) + st->dlogits_off;
      cnt = (size_t)st->lin.back().rows * st->classes;
      break;
    default:
      return fail(PD_EINVAL, "unknown tensor selector %d", what);
  }
  if (n != cnt) return fail(PD_EINVAL, "tensor has %zu elements, caller gave %zu", cnt, n);
  PD_HIP(st->sync_all());
  if (const int seq_rc = seq_check(st)) return seq_rc;
  if (!st->bf16 || (what == 0 && st->has_loss && layer == nl - 1)) {  // logits are fp32 in either mode
    PD_HIP(hipMemcpy(host_out, src, cnt * 4, hipMemcpyDeviceToHost));
    return PD_OK;
  }
  std::vector<uint16_t> tmp(cnt);
  PD_HIP(hipMemcpy(tmp.data(), src, cnt * 2, hipMemcpyDeviceToHost));
  for (size_t i = 0; i < cnt; ++i) {
    const uint32_t u = (uint32_t)tmp[i] << 16;
    memcpy(host_out + i, &u, 4);
  }
  return PD_OK;
}

int pd_stage_debug_write(pd_stage* st, int32_t what, int32_t mb_id, int32_t layer, const float* host_in, size_t n) {
  if (check_stage(st) || !host_in || mb_id < 0) return fail(PD_EINVAL, "bad argument");
  const int nl = (int)st->lin.size();
  char* dst = nullptr;
  size_t cnt = 0;
  bool as_f32 = !st->bf16;
  if (what == 0) {
    if (layer < 0 || layer >= nl) return fail(PD_EINVAL, "layer %d out of range", layer);
    if (st->lin[layer].kind == K_LSTM) return fail(PD_ESTATE, "an LSTM's stored state cannot be overwritten piecemeal");
    dst = st->out_of(st->stash_slot(mb_id), layer);
    cnt = (size_t)st->lin[layer].rows * st->lin[layer].out;
    if (st->has_loss && layer == nl - 1) as_f32 = true;  // logits
  } else if (what == 1) {
    dst = st->in_slot(mb_id);
    cnt = (size_t)st->lin.front().rows * st->lin.front().in;
  } else {
    return fail(PD_EINVAL, "unknown tensor selector %d", what);
  }
  if (n != cnt) return fail(PD_EINVAL, "tensor has %zu elements, caller gave %zu", cnt, n);
  PD_HIP(st->sync_all());
  if (const int seq_rc = seq_check(st)) return seq_rc;
  if (as_f32) {
    PD_HIP(hipMemcpy(dst, host_in, cnt * 4, hipMemcpyHostToDevice));
    return PD_OK;
  }
  std::vector<uint16_t> tmp(cnt);
  for (size_t i = 0; i < cnt; ++i) {  // round to nearest even (the values are expected to be bfloat16 already)
    uint32_t u;
    memcpy(&u, host_in + i, 4);
    u += 0x7fffu + ((u >> 16) & 1u);
    tmp[i] = (uint16_t)(u >> 16);
  }
  PD_HIP(hipMemcpy(dst, tmp.data(), cnt * 2, hipMemcpyHostToDevice));
  // a max-pooling layer that reads this tensor has recorded where ITS maxima were: pool again, so that its
  // routing words (and its stored output) belong to the values the tensor holds now.  Only for a minibatch whose
  // forward pass has run here (an input slot may be written before that, while an older minibatch still owns the
  // stash slot; the forward pass then records the routing itself).
  bool forward_done = false;
  for (const InFlight& f : st->in_flight) forward_done = forward_done || f.mb == mb_id;
  char* slot = st->stash_slot(mb_id);
  for (int li = 0; forward_done && li < nl; ++li) {
    const Layer& L = st->lin[li];
    if ((L.kind != K_POOL && L.kind != K_GPOOL) || (what == 0 ? L.src != layer : L.src >= 0)) continue;
    const char* a = L.src < 0 ? st->in_slot(mb_id) : st->out_of(slot, L.src);
    if (L.kind == K_POOL) {
      PD_HIP(pd::maxpool2x2_forward_bf16(st->stream, reinterpret_cast<const pd::bf16_t*>(a),
                                         reinterpret_cast<pd::bf16_t*>(st->out_of(slot, li)), pool_route(st, slot, L),
                                         st->B, L.ih, L.iw, L.ic));
    } else {
      const pd::PoolGeom g = {st->B, L.ih, L.iw, L.ic, L.kh, L.stride, L.ph, L.oh, L.ow};
      if (!pd::pool2d_routes(L.is_max, g)) continue;
      PD_HIP(pd::pool2d_forward_bf16(st->stream, true, reinterpret_cast<const pd::bf16_t*>(a),
                                     reinterpret_cast<pd::bf16_t*>(st->out_of(slot, li)), pool_route(st, slot, L), g));
    }
    PD_HIP(hipStreamSynchronize(st->stream));
  }
  return PD_OK;
}

// borrow_y (the pipeline driver only): y_dev is the consumer stage's input slot and stays intact until this stage's
// backward pass of the minibatch has run, so the last layer writes its output THERE and nowhere else: the hand-off
// costs no copy and no launch.  Otherwise y_dev receives a copy of the stored output.
static int forward_impl(pd_stage* st, int32_t mb_id, int32_t version, const void* x_dev, const int32_t* labels_dev,
                        void* y_dev, float* loss_dev, bool borrow_y) {
  if (check_stage(st)) return PD_EINVAL;
  if (version >= 0 && (version > st->latest || version <= st->latest - st->ring_depth))
    return fail(PD_ESTATE, "forward of minibatch %d asks for version %d, the stage holds %d..%d", mb_id, version,
                st->latest - st->ring_depth + 1 > 0 ? st->latest - st->ring_depth + 1 : 0, st->latest);
  if (!x_dev) return fail(PD_EINVAL, "x_dev is null");
  if (mb_id < 0) return fail(PD_EINVAL, "mb_id must be >= 0");
  if (st->has_loss && !labels_dev) return fail(PD_EINVAL, "labels_dev is required on a stage that ends in the loss");
  if (st->grad_pending) return fail(PD_ESTATE, "pd_update must follow pd_backward before the next forward");
  if ((int)st->in_flight.size() >= st->depth)
    return fail(PD_ESTATE, "%d minibatches already in flight (depth %d)", (int)st->in_flight.size(), st->depth);
  if (st->last_fwd >= 0 && mb_id != st->last_fwd + 1)
    return fail(PD_ESTATE, "forward of minibatch %d after %d: ids must be consecutive", mb_id, st->last_fwd);

  // slot safety (Section 4, intermediate state): what this forward pass writes must not belong to a minibatch in flight
  for (const InFlight& f : st->in_flight) {
    if (f.mb % st->depth == mb_id % st->depth)
      return fail(PD_ESTATE, "stash slot %d of minibatch %d is still held by minibatch %d", mb_id % st->depth, mb_id, f.mb);
    if (f.mb % st->in_depth == mb_id % st->in_depth)
      return fail(PD_ESTATE, "input slot %d of minibatch %d is still held by minibatch %d", mb_id % st->in_depth, mb_id, f.mb);
  }

  hipStream_t s = st->stream;
  // forward reads the latest version (or, under vertical sync, the one the minibatch carries) and stashes its id
  const int v = version >= 0 ? version : st->latest;
  char* in = st->in_slot(mb_id);
  char* slot = st->stash_slot(mb_id);
  const char* w = st->ring_slot(v);
  borrow_y = borrow_y && y_dev && !st->has_loss && st->lin.back().kind != K_LSTM;
  st->borrowed_out[mb_id % st->depth] = borrow_y ? static_cast<char*>(y_dev) : nullptr;
  if (x_dev != in) PD_HIP(pd::copy_bytes(s, x_dev, in, (size_t)st->lin.front().rows * st->lin.front().in * st->esz));
  PD_HIP(st->mark(-1, 0));
  int loss_splits = 0;                    // > 0: the last Linear layer left this many partial sums in the workspace
  const pd::bf16_t* loss_bias = nullptr;
  for (int li = 0; li < (int)st->lin.size(); ++li) {
    if (li > 0) PD_HIP(st->mark(0, li - 1));
    const Layer& L = st->lin[li];
    char* y = st->out_of(slot, li);
    const char* a = L.src < 0 ? in : st->out_of(slot, L.src);
    if (L.kind == K_LINEAR) {
      if (st->bf16) {
        const pd::bf16_t* wp = reinterpret_cast<const pd::bf16_t*>(w);
        const bool logits = st->has_loss && &L == &st->lin.back();  // logits go to the loss unrounded (fp32)
        if (logits && L.out <= pd::kFusedLossMaxClasses && !pd::linear_fwd_uses_big_tiles(L.rows, L.out) &&
            (size_t)L.rows * L.out * 4 <= st->ws_bytes) {
          // leave the split-K partial sums: the loss kernel adds them up, writes the logits and takes the loss
          PD_HIP(pd::gemm_partial_bf16(s, false, reinterpret_cast<const pd::bf16_t*>(a), 0, wp + L.w_off, L.rows,
                                       L.out, L.in, st->ws, st->ws_bytes, &loss_splits));
          loss_bias = wp + L.b_off;
          continue;
        }
        PD_HIP(pd::linear_fwd_bf16(s, reinterpret_cast<const pd::bf16_t*>(a), wp + L.w_off, wp + L.b_off,
                                   reinterpret_cast<pd::bf16_t*>(y), logits ? reinterpret_cast<float*>(y) : nullptr,
                                   L.rows, L.out, L.in, L.relu, st->ws, st->ws_bytes));
      } else {
        const float* wp = reinterpret_cast<const float*>(w);
        PD_HIP(pd::linear_fwd_f32(s, reinterpret_cast<const float*>(a), wp + L.w_off, wp + L.b_off,
                                  reinterpret_cast<float*>(y), L.rows, L.out, L.in, L.relu));
      }
    } else if (L.kind == K_LSTM) {
      // input projection of the whole sequence in one GEMM (bias folded in, fp32), then the recurrence: per
      // step one skinny GEMM h_{t-1} W_hh^T left as partial sums and one cell kernel that adds them up
      const pd::bf16_t* wp = reinterpret_cast<const pd::bf16_t*>(w);
      const pd::bf16_t* wih = wp + L.w_off;
      const pd::bf16_t* whh = wih + (size_t)4 * L.out * L.in;
      const int B = st->B, H = L.out;
      float* gates = reinterpret_cast<float*>(slot + L.g_off);
      float* cbuf = reinterpret_cast<float*>(slot + L.c_off);
      pd::bf16_t* hbuf = reinterpret_cast<pd::bf16_t*>(slot + L.y_off);
      PD_HIP(pd::linear_fwd_bf16(s, reinterpret_cast<const pd::bf16_t*>(a), wih, wp + L.b_off, nullptr, gates, L.rows,
                                 4 * H, L.in, false, st->ws, st->ws_bytes));
      if (seq_wanted(st, s, B, H, L.T)) {  // all time steps in one launch
        PD_HIP(seq_chain_enter(s));
        PD_HIP(pd::lstm_seq_forward(s, gates, hbuf, whh, cbuf, st->seq_sync, B, H, L.T, g_seq_spin_limit, g_seq_starve));
        PD_HIP(seq_chain_leave(s));
        st->seq_used = true;
      } else {
        for (int t = 0; t < L.T; ++t) {
          if (t == 0)
            PD_HIP(pd::lstm_cell_forward(s, gates, nullptr, 0, cbuf, cbuf + (size_t)B * H, hbuf + (size_t)B * H, B, H));
          else
            PD_HIP(pd::lstm_step_forward(s, gates + (size_t)t * B * 4 * H, hbuf + (size_t)t * B * H, whh,
                                         cbuf + (size_t)t * B * H, cbuf + (size_t)(t + 1) * B * H,
                                         hbuf + (size_t)(t + 1) * B * H, B, H));
        }
      }
    } else if (L.kind == K_CONV) {
      const pd::bf16_t* wp = reinterpret_cast<const pd::bf16_t*>(w);
      const pd::ConvGeom g = {st->B, L.ih, L.iw, L.ic, L.oh, L.ow, L.oc, L.kh, L.kw, L.stride, L.ph, L.pw};
      const pd::ConvEpilogue ep = {wp + L.b_off, nullptr, L.relu ? 1 : 0, reinterpret_cast<pd::bf16_t*>(y)};
      PD_HIP(pd::conv_forward_bf16(s, reinterpret_cast<const pd::bf16_t*>(a), wp + L.w_off, g, ep));
    } else if (L.kind == K_POOL) {
      PD_HIP(pd::maxpool2x2_forward_bf16(s, reinterpret_cast<const pd::bf16_t*>(a), reinterpret_cast<pd::bf16_t*>(y),
                                         pool_route(st, slot, L), st->B, L.ih, L.iw, L.ic));
    } else if (L.kind == K_GPOOL) {
      const pd::PoolGeom g = {st->B, L.ih, L.iw, L.ic, L.kh, L.stride, L.ph, L.oh, L.ow};
      PD_HIP(pd::pool2d_forward_bf16(s, L.is_max, reinterpret_cast<const pd::bf16_t*>(a),
                                     reinterpret_cast<pd::bf16_t*>(y),
                                     pd::pool2d_routes(L.is_max, g) ? pool_route(st, slot, L) : nullptr, g));
    } else {  // K_CONCAT: assemble the block's output from the branch outputs, branch 0 first
      const size_t pixels = (size_t)st->B * L.oh * L.ow;
      for (int b = 0; b < L.nbr; ++b)
        PD_HIP(pd::copy_channels_bf16(s, reinterpret_cast<const pd::bf16_t*>(st->out_of(slot, L.b_last[b])), L.b_c[b], 0,
                                      reinterpret_cast<pd::bf16_t*>(y), L.oc, L.b_coff[b], nullptr, pixels, L.b_c[b]));
    }
  }
  char* a = st->out_of(slot, (int)st->lin.size() - 1);
  if (st->has_loss) {
    if (loss_splits > 0)
      PD_HIP(pd::softmax_xent_partials(s, st->ws, loss_splits, loss_bias, reinterpret_cast<float*>(a), labels_dev,
                                       slot + st->dlogits_off, st->row_loss, loss_dev, st->lin.back().rows, st->classes,
                                       st->bf16));
    else
      PD_HIP(pd::softmax_xent(s, reinterpret_cast<const float*>(a), labels_dev, slot + st->dlogits_off, st->row_loss,
                              loss_dev, st->lin.back().rows, st->classes, st->bf16));
  }
  if (y_dev && !borrow_y)
    PD_HIP(pd::copy_bytes(s, a, y_dev, (size_t)st->lin.back().rows * st->lin.back().out * (st->has_loss ? 4 : st->esz)));
  PD_HIP(st->mark(0, (int)st->lin.size() - 1));  // (the loss and the copy of the output count for the last layer)
  if (st->profiling) ++st->prof_ops[0];
  if (st->stream_b) PD_HIP(hipEventRecord(st->ev_fwd[mb_id % st->depth], st->stream));
  st->in_flight.push_back({mb_id, v});
  st->last_fwd = mb_id;
  st->log_op(PD_OP_F, mb_id, v);
  return PD_OK;
}

int pd_forward(pd_stage* st, int32_t mb_id, const void* x_dev, const int32_t* labels_dev, void* y_dev,
               float* loss_dev) {
  return forward_impl(st, mb_id, -1, x_dev, labels_dev, y_dev, loss_dev, false);
}

int pd_forward_versioned(pd_stage* st, int32_t mb_id, int32_t version, const void* x_dev, const int32_t* labels_dev,
                         void* y_dev, float* loss_dev) {
  return forward_impl(st, mb_id, version, x_dev, labels_dev, y_dev, loss_dev, false);
}

// The pipeline driver's variants of the gradient hand-off between two stages:
//   dy_is_dz    dy_dev already is dL/d(pre-activation) of this stage's last layer (the consumer stage applied this
//               stage's ReLU mask when it stored the gradient) and stays intact until pd_update: it is used where it
//               lies, with no masking or copying launch;
//   mask_input  the producer stage ends in a ReLU: dL/d(input) is stored with that ReLU's mask applied, taken from this
//               stage's own input slot, which holds the producer's output.
static int backward_impl(pd_stage* st, int32_t mb_id, const void* dy_dev, void* dx_dev, bool dy_is_dz, bool mask_input) {
  if (check_stage(st)) return PD_EINVAL;
  if (st->grad_pending) return fail(PD_ESTATE, "previous gradient not yet consumed by pd_update");
  if (st->in_flight.empty()) return fail(PD_ESTATE, "no minibatch in flight");
  if (st->in_flight.front().mb != mb_id)
    return fail(PD_ESTATE, "backward of minibatch %d, but the oldest in flight is %d", mb_id, st->in_flight.front().mb);
  if (st->has_loss && dy_dev) return fail(PD_EINVAL, "dy_dev must be NULL on a stage that ends in the loss");
  if (!st->has_loss && !dy_dev) return fail(PD_EINVAL, "dy_dev is null");

  hipStream_t s = st->bstream();
  if (st->stream_b) {
    // Backward lane: this pass needs its minibatch's forward pass, and it overwrites the set of gradient buffers that
    // the update before the last one read (exactly one update lies between two backward passes).  It therefore starts
    // as soon as that update is done and runs next to the forward pass behind it.  (Holding it back until that forward
    // pass is done, so that it runs next to the following update instead, was slower: VGG16 classifier stage 0.522
    // against 0.500 ms per step.)
    PD_HIP(hipStreamWaitEvent(s, st->ev_fwd[mb_id % st->depth], 0));
    if (st->n_upd >= 2) PD_HIP(hipStreamWaitEvent(s, st->ev_upd[st->n_upd & 1], 0));
    st->dz = st->dz_base + (size_t)st->bwd_set * st->dz_set_bytes;
    st->part = st->part_base + (size_t)st->bwd_set * st->part_set_bytes;
    st->bwd_set ^= 1;
  }
  float* const ws = st->ws_b ? st->ws_b : st->ws;  // (the lane's own split-K workspace: a forward pass may be running)
  const int v = st->in_flight.front().version;  // the version this minibatch's forward read
  const char* w = st->ring_slot(v);
  char* slot = st->stash_slot(mb_id);
  const int nl = (int)st->lin.size();
  const Layer& last = st->lin.back();
  // `cur` = dL/d(output of layer l) with layer l's own ReLU mask already applied.  Linear layers keep it in
  // their own buffer until pd_update (the weight gradient is formed there); conv/pool layers ping-pong.
  int pp_next = 0;
  auto buffer_for = [&](int l) -> char* {
    if (st->lin[l].kind == K_LINEAR) return st->dz + st->lin[l].dz_off;  // (an LSTM's own buffer holds dG)
    char* b = st->pp + (size_t)pp_next * st->pp_bytes;
    pp_next ^= 1;
    return b;
  };
  const char* cur;
  PD_HIP(st->mark(-1, 0));
  if (st->has_loss) {
    cur = slot + st->dlogits_off;
  } else if (dy_is_dz) {
    cur = static_cast<const char*>(dy_dev);
  } else {
    char* b = buffer_for(nl - 1);
    const size_t n = (size_t)last.rows * last.out;
    if (last.relu) PD_HIP(pd::relu_mask(s, dy_dev, st->out_of(slot, nl - 1), b, n, st->bf16));
    else PD_HIP(pd::copy_bytes(s, dy_dev, b, n * st->esz));
    cur = b;
  }
  int prof_l = nl - 1;  // the layer whose kernels were enqueued since the last mark
  for (int l = nl - 1; l >= 0; --l) {
    if (l < nl - 1) PD_HIP(st->mark(1, prof_l));
    prof_l = l;
    const Layer& L = st->lin[l];
    if (L.kind == K_CONCAT) {
      // `cur` is dL/d(block output).  Split it into one contiguous tensor per branch, applying the ReLU mask of
      // the branch's last layer on the way; the branches are then walked one after the other (they sit at the
      // indices below this one), each starting from its own slice.
      const size_t pixels = (size_t)st->B * L.oh * L.ow;
      for (int b = 0; b < L.nbr; ++b) {
        const Layer& E = st->lin[L.b_last[b]];
        const char* mask = E.relu ? st->out_of(slot, L.b_last[b]) : nullptr;
        PD_HIP(pd::copy_channels_bf16(s, reinterpret_cast<const pd::bf16_t*>(cur), L.oc, L.b_coff[b],
                                      reinterpret_cast<pd::bf16_t*>(st->blk_dy + E.bdy_off), L.b_c[b], 0,
                                      reinterpret_cast<const pd::bf16_t*>(mask), pixels, L.b_c[b]));
      }
      continue;
    }
    if (L.br_last) cur = st->blk_dy + L.bdy_off;
    const char* x = L.src < 0 ? st->in_slot(mb_id) : st->out_of(slot, L.src);
    if (L.kind == K_CONV) {  // weight-gradient partial sums; pd_update reduces them and applies the update
      const pd::ConvGeom g = {st->B, L.ih, L.iw, L.ic, L.oh, L.ow, L.oc, L.kh, L.kw, L.stride, L.ph, L.pw};
      PD_HIP(pd::conv_wgrad_partial_bf16(s, reinterpret_cast<const pd::bf16_t*>(cur),
                                         reinterpret_cast<const pd::bf16_t*>(x),
                                         reinterpret_cast<float*>(st->part + L.part_off), L.splits, g));
    }
    if (L.kind == K_LSTM) {  // back-propagation through time: leaves dL/d(gate pre-activations) for every step
      const pd::bf16_t* wp = reinterpret_cast<const pd::bf16_t*>(w);
      const pd::bf16_t* whh = wp + L.w_off + (size_t)4 * L.out * L.in;
      const int B = st->B, H = L.out;
      pd::bf16_t* dG = reinterpret_cast<pd::bf16_t*>(st->dz + L.dz_off);
      float* dc = reinterpret_cast<float*>(st->dz + L.dc_off);
      const float* gates = reinterpret_cast<const float*>(slot + L.g_off);
      const float* cbuf = reinterpret_cast<const float*>(slot + L.c_off);
      const pd::bf16_t* dh_out = reinterpret_cast<const pd::bf16_t*>(cur);
      PD_HIP(pd::fill_zero(s, dc, (size_t)B * H * 4));
      // dh_{t} needs da_{t+1} W_hh: with W_hh^T laid out [H][4H] that is the same reduction-contiguous product as
      // in the forward pass, so transpose once per backward pass instead of transposing tiles at every step
      pd::bf16_t* whh_t = reinterpret_cast<pd::bf16_t*>(st->wt);
      PD_HIP(pd::transpose_bf16(s, whh, whh_t, 4 * H, H));
      if (seq_wanted(st, s, B, H, L.T)) {  // all time steps in one launch (the cell gradient stays in registers)
        PD_HIP(seq_chain_enter(s));
        PD_HIP(pd::lstm_seq_backward(s, dh_out, dG, whh_t, gates, cbuf, st->seq_sync + pd::kSeqSyncWords, B, H, L.T,
                                     g_seq_spin_limit, g_seq_starve));
        PD_HIP(seq_chain_leave(s));
        st->seq_used = true;
      } else {
        for (int t = L.T - 1; t >= 0; --t) {
          if (t == L.T - 1)
            PD_HIP(pd::lstm_cell_backward(s, dh_out + (size_t)t * B * H, nullptr, 0, dc, gates + (size_t)t * B * 4 * H,
                                          cbuf + (size_t)(t + 1) * B * H, cbuf + (size_t)t * B * H,
                                          dG + (size_t)t * B * 4 * H, B, H));
          else
            PD_HIP(pd::lstm_step_backward(s, dh_out + (size_t)t * B * H, dG + (size_t)(t + 1) * B * 4 * H, whh_t, dc,
                                          gates + (size_t)t * B * 4 * H, cbuf + (size_t)(t + 1) * B * H,
                                          cbuf + (size_t)t * B * H, dG + (size_t)t * B * 4 * H, B, H));
        }
      }
    }
    char* out;
    const char* mask = nullptr;
    // where the block's summed input gradient goes (first layer of a branch): null = nobody wants it
    const Layer* blk = L.block >= 0 ? &st->lin[L.block] : nullptr;
    const bool blk_wanted = blk && (blk->blk_src >= 0 || dx_dev);
    if (L.br_first) {
      if (!blk_wanted) {
        if (l == 0) break;
        continue;
      }
      out = st->blk_dx + L.bdx_off;  // unmasked: the mask of the block's producer is applied to the sum
    } else if (L.src >= 0) {
      out = buffer_for(L.src);
      if (st->lin[L.src].relu) mask = st->out_of(slot, L.src);
    } else {
      if (!dx_dev) break;
      out = static_cast<char*>(dx_dev);
      if (mask_input) mask = st->in_slot(mb_id);
    }
    if (L.kind == K_LINEAR) {
      if (st->bf16) {
        const pd::bf16_t* wp = reinterpret_cast<const pd::bf16_t*>(w);
        PD_HIP(pd::linear_dgrad_bf16(s, reinterpret_cast<const pd::bf16_t*>(cur), wp + L.w_off,
                                     reinterpret_cast<const pd::bf16_t*>(mask), reinterpret_cast<pd::bf16_t*>(out),
                                     L.rows, L.out, L.in, ws, st->ws_bytes));
      } else {
        const float* wp = reinterpret_cast<const float*>(w);
        PD_HIP(pd::linear_dgrad_f32(s, reinterpret_cast<const float*>(cur), wp + L.w_off,
                                    reinterpret_cast<const float*>(mask), reinterpret_cast<float*>(out), L.rows, L.out,
                                    L.in));
      }
    } else if (L.kind == K_LSTM) {
      const pd::bf16_t* wp = reinterpret_cast<const pd::bf16_t*>(w);
      const pd::bf16_t* wih = wp + L.w_off;
      const pd::bf16_t* whh = wih + (size_t)4 * L.out * L.in;
      PD_HIP(pd::linear_dgrad_bf16(s, reinterpret_cast<const pd::bf16_t*>(st->dz + L.dz_off), wih,
                                   reinterpret_cast<const pd::bf16_t*>(mask), reinterpret_cast<pd::bf16_t*>(out), L.rows,
                                   4 * L.out, L.in, ws, st->ws_bytes));
      (void)whh;
    } else if (L.kind == K_CONV) {
      const pd::bf16_t* wp = reinterpret_cast<const pd::bf16_t*>(w);
      const pd::ConvGeom g = {st->B, L.ih, L.iw, L.ic, L.oh, L.ow, L.oc, L.kh, L.kw, L.stride, L.ph, L.pw};
      const pd::ConvEpilogue ep = {nullptr, reinterpret_cast<const pd::bf16_t*>(mask), 0,
                                   reinterpret_cast<pd::bf16_t*>(out)};
      PD_HIP(pd::conv_dgrad_bf16(s, reinterpret_cast<const pd::bf16_t*>(cur), wp + L.w_off,
                                 reinterpret_cast<pd::bf16_t*>(st->wt), g, ep));
    } else if (L.kind == K_POOL) {
      PD_HIP(pd::maxpool2x2_backward_routed_bf16(s, pool_route(st, slot, L), reinterpret_cast<const pd::bf16_t*>(cur),
                                                 reinterpret_cast<pd::bf16_t*>(out), st->B, L.ih, L.iw, L.ic,
                                                 mask != nullptr));
    } else {  // K_GPOOL (the pooling kernels take the mask as "x > 0", x being the stored output of the producer)
      const pd::PoolGeom g = {st->B, L.ih, L.iw, L.ic, L.kh, L.stride, L.ph, L.oh, L.ow};
      if (pd::pool2d_routes(L.is_max, g))
        PD_HIP(pd::pool2d_backward_routed_bf16(s, pool_route(st, slot, L), reinterpret_cast<const pd::bf16_t*>(cur),
                                               reinterpret_cast<pd::bf16_t*>(out), g, mask != nullptr));
      else
        PD_HIP(pd::pool2d_backward_bf16(s, L.is_max, reinterpret_cast<const pd::bf16_t*>(x),
                                        reinterpret_cast<const pd::bf16_t*>(st->out_of(slot, l)),
                                        reinterpret_cast<const pd::bf16_t*>(cur), reinterpret_cast<pd::bf16_t*>(out), g,
                                        mask != nullptr));
    }
    cur = out;
    if (L.br_first && l == blk->b_first[0]) {
      // every branch has left its input gradient: add them up in branch order, apply the producer's ReLU mask
      const pd::bf16_t* parts[pd::kMaxBranches];
      for (int b = 0; b < blk->nbr; ++b)
        parts[b] = reinterpret_cast<const pd::bf16_t*>(st->blk_dx + st->lin[blk->b_first[b]].bdx_off);
      char* sum_out;
      const char* sum_mask = nullptr;
      if (blk->blk_src >= 0) {
        sum_out = buffer_for(blk->blk_src);
        if (st->lin[blk->blk_src].relu) sum_mask = st->out_of(slot, blk->blk_src);
      } else {
        sum_out = static_cast<char*>(dx_dev);
        if (mask_input) sum_mask = st->in_slot(mb_id);
      }
      PD_HIP(pd::sum_tensors_bf16(s, parts, blk->nbr, reinterpret_cast<const pd::bf16_t*>(sum_mask),
                                  reinterpret_cast<pd::bf16_t*>(sum_out), blk->blk_in_elems));
      cur = sum_out;
    }
  }
  PD_HIP(st->mark(1, prof_l));
  if (st->profiling) ++st->prof_ops[1];
  if (st->stream_b) PD_HIP(hipEventRecord(st->ev_bwd, s));
  st->in_flight.pop_front();  // stash slot released; the factored gradient stays valid until pd_update
  st->grad_pending = true;
  st->pending_mb = mb_id;
  st->borrowed_dz = (dy_is_dz && !st->has_loss) ? static_cast<const char*>(dy_dev) : nullptr;
  st->log_op(PD_OP_B, mb_id, v);
  return PD_OK;
}

int pd_backward(pd_stage* st, int32_t mb_id, const void* dy_dev, void* dx_dev) {
  return backward_impl(st, mb_id, dy_dev, dx_dev, false, false);
}

}  // extern "C"

namespace {

// The kernels of U for the pending minibatch of `st`.  grad_only = false: weight gradient fused with the step of the
// stage's rule into ring slot `nv`.  grad_only = true (a replica of a replicated stage): the same kernels leave the
// fp32 gradient in st->gradbuf, laid out like a parameter set, and change nothing else.
int run_update_kernels(pd_stage* st, int nv, bool grad_only) {
  hipStream_t s = st->stream;
  if (st->stream_b) PD_HIP(hipStreamWaitEvent(s, st->ev_bwd, 0));  // the pending gradient was formed on the backward lane
  const int mb = st->pending_mb;
  char* slot = st->stash_slot(mb);
  const int nl = (int)st->lin.size();
  const pd::UpdateRule rule = grad_only ? pd::UpdateRule{0.f, 0.f, 0.f, pd::kRuleGradOnly} : st->rule;
  float* const w32 = grad_only ? st->gradbuf : st->master;  // bf16 mode: where the fp32 result of a kernel goes
  pd::WgradBatch batch;
  batch.count = 0; batch.M = st->B; batch.rule = rule;
  PD_HIP(st->mark(-1, 0));
  // Last layer first: the forward pass that follows the update in the 1F1B order reads the first layer's new ring
  // copy first, and finds part of it still cached if that layer was written last.  VGG16 classifier stage on
  // MI355X: forward product of the 25088 x 4096 layer 57.7 -> 36.5 us, update kernel 372 -> 378 us, step 0.555 ->
  // 0.546 ms; convolution, LSTM and branched-block stages unchanged.
  for (int l = nl - 1; l >= 0; --l) {
    const Layer& L = st->lin[l];
    if (!L.n_w) continue;  // pooling, concatenation
    if (L.kind == K_CONV) {  // partial sums left by pd_backward -> step into the next ring slot
      pd::bf16_t* ro = reinterpret_cast<pd::bf16_t*>(st->ring_slot(nv));
      PD_HIP(pd::wgrad_reduce_update(s, reinterpret_cast<const float*>(st->part + L.part_off), L.splits, 0, L.n_w,
                                     (int)L.n_b, w32 + L.w_off, st->mom + L.w_off, ro + L.w_off,
                                     w32 + L.b_off, st->mom + L.b_off, ro + L.b_off, rule));
      PD_HIP(st->mark(2, l));
      continue;
    }
    const char* dz = (st->has_loss && l == nl - 1) ? slot + st->dlogits_off
                     : (l == nl - 1 && st->borrowed_dz && L.kind == K_LINEAR) ? st->borrowed_dz : st->dz + L.dz_off;
    const char* x = L.src < 0 ? st->in_slot(mb) : st->out_of(slot, L.src);
    if (st->bf16 && L.splits > 0) {  // many rows: partial sums over row ranges, then reduce + update
      pd::bf16_t* ro = reinterpret_cast<pd::bf16_t*>(st->ring_slot(nv));
      const int n_out = L.kind == K_LSTM ? 4 * L.out : L.out;
      float* part = reinterpret_cast<float*>(st->part + L.part_off);
      const size_t n_w1 = (size_t)n_out * L.in, o2 = L.w_off + n_w1;
      const pd::bf16_t* dzp = reinterpret_cast<const pd::bf16_t*>(dz);
      const pd::bf16_t* h_prev = reinterpret_cast<const pd::bf16_t*>(slot + L.y_off);  // LSTM: hidden states, shifted
      if (grad_only) {
        PD_HIP(pd::linear_wgrad_big_bf16(s, dzp, reinterpret_cast<const pd::bf16_t*>(x), w32 + L.w_off, w32 + L.b_off,
                                         L.rows, n_out, L.in, st->ws, st->ws_bytes));
        if (L.kind == K_LSTM)
          PD_HIP(pd::linear_wgrad_big_bf16(s, dzp, h_prev, w32 + o2, nullptr, L.rows, n_out, L.out, st->ws,
                                           st->ws_bytes));
        PD_HIP(st->mark(2, l));
        continue;
      }
      PD_HIP(pd::linear_wgrad_update_big_bf16(s, dzp, reinterpret_cast<const pd::bf16_t*>(x), part, L.rows, n_out, L.in,
                                              st->master + L.w_off, st->mom + L.w_off, ro + L.w_off,
                                              st->master + L.b_off, st->mom + L.b_off, ro + L.b_off, rule,
                                              st->ws, st->ws_bytes));
      if (L.kind == K_LSTM) {
        float* part2 = reinterpret_cast<float*>(st->part + L.part2_off);
        PD_HIP(pd::linear_wgrad_update_big_bf16(s, dzp, h_prev, part2, L.rows, n_out, L.out, st->master + o2,
                                                st->mom + o2, ro + o2, nullptr, nullptr, nullptr, rule, st->ws,
                                                st->ws_bytes));
      }
      PD_HIP(st->mark(2, l));
    } else if (st->bf16) {
      pd::bf16_t* ro = reinterpret_cast<pd::bf16_t*>(st->ring_slot(nv));
      auto flush_if_full = [&]() -> hipError_t {
        if (batch.count < pd::kMaxWgradLayers) return hipSuccess;
        hipError_t e = pd::linear_wgrad_update_bf16(s, batch);
        batch.count = 0;
        if (e == hipSuccess) e = st->mark(3, -1);
        return e;
      };
      pd::WgradLayer& W = batch.layer[batch.count++];
      W.dz = reinterpret_cast<const pd::bf16_t*>(dz); W.x = reinterpret_cast<const pd::bf16_t*>(x);
      const pd::bf16_t* rin = reinterpret_cast<const pd::bf16_t*>(st->ring_slot(st->latest));
      const bool split = L.split_master && !grad_only;
      W.master_w = w32 + L.w_off; W.mom_w = st->mom + L.w_off; W.ring_w = ro + L.w_off;
      W.ring_in = split ? rin + L.w_off : nullptr; W.rem_w = split ? st->rem + L.w_off : nullptr;
      W.master_b = w32 + L.b_off; W.mom_b = st->mom + L.b_off; W.ring_b = ro + L.b_off;
      W.M = L.rows; W.N = L.kind == K_LSTM ? 4 * L.out : L.out; W.K = L.in; W.tile_end = 0;
      PD_HIP(flush_if_full());
      if (L.kind == K_LSTM) {  // second matrix: W_hh, whose "input" is the hidden sequence shifted by one step
        const size_t o2 = L.w_off + (size_t)4 * L.out * L.in;
        pd::WgradLayer& V = batch.layer[batch.count++];
        V.dz = reinterpret_cast<const pd::bf16_t*>(dz);
        V.x = reinterpret_cast<const pd::bf16_t*>(slot + L.y_off);
        V.master_w = w32 + o2; V.mom_w = st->mom + o2; V.ring_w = ro + o2;
        V.ring_in = split ? rin + o2 : nullptr; V.rem_w = split ? st->rem + o2 : nullptr;
        V.master_b = nullptr; V.mom_b = nullptr; V.ring_b = nullptr;
        V.M = L.rows; V.N = 4 * L.out; V.K = L.out; V.tile_end = 0;
        PD_HIP(flush_if_full());
      }
    } else {
      const float* wi = reinterpret_cast<const float*>(st->ring_slot(st->latest));
      float* wo = grad_only ? st->gradbuf : reinterpret_cast<float*>(st->ring_slot(nv));
      PD_HIP(pd::linear_wgrad_update_f32(s, reinterpret_cast<const float*>(dz), reinterpret_cast<const float*>(x),
                                         wi + L.w_off, wo + L.w_off, st->mom + L.w_off, wi + L.b_off, wo + L.b_off,
                                         st->mom + L.b_off, L.rows, L.out, L.in, rule));
      PD_HIP(st->mark(2, l));
    }
  }
  if (batch.count) {  // all Linear layers of the stage in one launch
    PD_HIP(pd::linear_wgrad_update_bf16(s, batch));
    PD_HIP(st->mark(3, -1));
  }
  if (st->profiling) ++st->prof_ops[2];
  return PD_OK;
}

// Slot safety of the version ring (Section 3.4: a minibatch's backward pass reads the weights its forward pass read):
// version nv goes into the slot that held version nv - ring_depth, so no minibatch in flight may still refer to that
// version or an older one.  The 1F1B order guarantees it; a caller that asked pd_forward_versioned for the oldest
// version held and then lets further updates pass does not.
int ring_slot_is_free(const pd_stage* st, int nv) {
  for (const InFlight& f : st->in_flight)
    if (f.version <= nv - st->ring_depth)
      return fail(PD_ESTATE, "the update to version %d would overwrite ring slot %d, which holds version %d, read by the "
                  "forward pass of in-flight minibatch %d", nv, nv % st->ring_depth, f.version, f.mb);
  return PD_OK;
}

}  // namespace

extern "C" {

int pd_update(pd_stage* st) {
  if (check_stage(st)) return PD_EINVAL;
  if (st->n_replicas > 1) return fail(PD_ESTATE, "replicated stage: its replicas are updated together by pd_update_replicated");
  if (!st->grad_pending) return fail(PD_ESTATE, "no pending gradient");
  const int nv = st->latest + 1;
  if (ring_slot_is_free(st, nv)) return PD_ESTATE;
  const int rc = run_update_kernels(st, nv, false);
  if (rc != PD_OK) return rc;
  if (st->stream_b) {
    PD_HIP(hipEventRecord(st->ev_upd[st->n_upd & 1], st->stream));
    ++st->n_upd;
  }
  st->latest = nv;
  st->grad_pending = false;
  st->log_op(PD_OP_U, st->pending_mb, nv);
  return PD_OK;
}

// Replicated stage (Section 3.3; Section 4 "Data Parallelism"): every replica with a pending gradient forms it on
// its own stream; the primary's stream waits for all replicas, sums the gradients in replica order and takes the one
// step on the shared parameter state; every replica's stream then waits for that step.
int pd_update_replicated(pd_stage* const* replicas, int32_t n_replicas) {
  if (!replicas || n_replicas < 1) return fail(PD_EINVAL, "need the replicas of the stage");
  pd_stage* p0 = replicas[0];
  if (check_stage(p0)) return PD_EINVAL;
  if (p0->primary) return fail(PD_EINVAL, "replicas[0] must be the primary");
  if (p0->n_replicas < 2) return fail(PD_EINVAL, "the stage is not configured as replicated");
  if (n_replicas != p0->n_replicas || (int)p0->secondaries.size() + 1 != n_replicas)
    return fail(PD_EINVAL, "the stage is configured for %d replicas, %zu exist, %d were passed", p0->n_replicas,
                p0->secondaries.size() + 1, n_replicas);
  for (int q = 1; q < n_replicas; ++q)
    if (replicas[q] != p0->secondaries[q - 1]) return fail(PD_EINVAL, "replicas must be passed in the order they were created (entry %d)", q);
  pd::ReplicaGrads grads;
  grads.count = 0;
  for (int q = 0; q < n_replicas; ++q) {
    if (replicas[q]->latest != p0->latest) return fail(PD_ESTATE, "replica %d is at another weight version", q);
    if (replicas[q]->grad_pending) grads.g[grads.count++] = replicas[q]->gradbuf;
  }
  if (!grads.count) return fail(PD_ESTATE, "no pending gradient on any replica");
  const int nv = p0->latest + 1;
  for (int q = 0; q < n_replicas; ++q)
    if (ring_slot_is_free(replicas[q], nv)) return PD_ESTATE;
  for (int q = 0; q < n_replicas; ++q) {
    pd_stage* r = replicas[q];
    if (r->grad_pending) {
      const int rc = run_update_kernels(r, nv, true);
      if (rc != PD_OK) return rc;
    }
    if (q > 0 && r->stream != p0->stream) {  // also a replica without a gradient may still be reading old versions
      PD_HIP(hipEventRecord(r->ev_rep, r->stream));
      PD_HIP(hipStreamWaitEvent(p0->stream, r->ev_rep, 0));
    }
  }
  if (p0->bf16) {
    PD_HIP(pd::replica_sum_update(p0->stream, grads, p0->master, p0->master, p0->mom,
                                  reinterpret_cast<pd::bf16_t*>(p0->ring_slot(nv)), p0->p_pad, p0->rule));
  } else {
    PD_HIP(pd::replica_sum_update(p0->stream, grads, reinterpret_cast<const float*>(p0->ring_slot(p0->latest)),
                                  reinterpret_cast<float*>(p0->ring_slot(nv)), p0->mom, nullptr, p0->p_pad, p0->rule));
  }
  PD_HIP(hipEventRecord(p0->ev_rep, p0->stream));
  for (int q = 0; q < n_replicas; ++q) {
    pd_stage* r = replicas[q];
    if (q > 0 && r->stream != p0->stream) PD_HIP(hipStreamWaitEvent(r->stream, p0->ev_rep, 0));
    r->latest = nv;
    if (r->grad_pending) r->log_op(PD_OP_U, r->pending_mb, nv);
    r->grad_pending = false;
  }
  return PD_OK;
}

// ---- layer profiler (Section 3.2, "Profiling the DNN model") ---------------------------------------------
int pd_stage_profile(pd_stage* st, int32_t enable) {
  if (check_stage(st)) return PD_EINVAL;
  if (enable && st->stream_b) return fail(PD_ESTATE, "the layer profiler times one stream: not for a stage with a backward stream of its own");
  if (enable) {
    for (const pd_stage::Mark& m : st->marks) st->mark_pool.push_back(m.ev);
    st->marks.clear();
    st->prof_ops[0] = st->prof_ops[1] = st->prof_ops[2] = 0;
  }
  st->profiling = enable != 0;
  return PD_OK;
}

int pd_stage_profile_read(pd_stage* st, pd_layer_profile* out, size_t cap, size_t* n_out) {
  if (check_stage(st)) return PD_EINVAL;
  const int nl = (int)st->lin.size();
  // profile units: a layer outside any block is one unit; a block of branches (its branch layers and the
  // concatenation that closes it) is one unit, because a pipeline can only be cut between units
  std::vector<int> unit_of(nl, 0);
  std::vector<pd_layer_profile> units;
  for (int l = 0; l < nl; ++l) {
    const Layer& L = st->lin[l];
    const int closing = L.kind == K_CONCAT ? l : L.block;  // index of the K_CONCAT layer, -1 outside blocks
    if (closing >= 0 && !units.empty() && units.back().last_layer == closing) {
      unit_of[l] = (int)units.size() - 1;
      continue;
    }
    pd_layer_profile u;
    memset(&u, 0, sizeof u);
    u.first_layer = l;
    u.last_layer = closing >= 0 ? closing : l;
    unit_of[l] = (int)units.size();
    units.push_back(u);
  }
  for (int l = 0; l < nl; ++l) {
    const Layer& L = st->lin[l];
    pd_layer_profile& u = units[unit_of[l]];
    u.param_bytes += 4.0 * (double)(L.n_w + L.n_b);  // fp32: what replicas of the stage would exchange
    if (l == u.last_layer) {
      const bool logits = st->has_loss && l == nl - 1;
      u.act_bytes = (double)L.rows * L.out * (logits ? 4 : st->esz);
    }
  }
  if (n_out) *n_out = units.size();
  if (units.size() > cap) return fail(PD_ENOMEM, "profile has %zu units, capacity %zu", units.size(), cap);
  if (!out) return fail(PD_EINVAL, "out is null");
  PD_HIP(st->sync_all());
  if (const int seq_rc = seq_check(st)) return seq_rc;
  // parameters updated by the one multi-layer launch: its time is shared out by parameter count (the launch
  // streams master weights and momentum once, so its time is proportional to them)
  double batch_params = 0;
  for (const Layer& L : st->lin)
    if (L.n_w && L.kind != K_CONV && st->bf16 && L.splits == 0) batch_params += (double)(L.n_w + L.n_b);
  for (size_t i = 1; i < st->marks.size(); ++i) {
    const pd_stage::Mark& m = st->marks[i];
    if (m.phase < 0) continue;  // start of an op: the time since the previous mark is not this stage's work
    float ms = 0.f;
    PD_HIP(hipEventElapsedTime(&ms, st->marks[i - 1].ev, m.ev));
    if (m.phase == 3) {
      for (int l = 0; l < nl; ++l) {
        const Layer& L = st->lin[l];
        if (L.n_w && L.kind != K_CONV && st->bf16 && L.splits == 0)
          units[unit_of[l]].upd_ms += ms * (double)(L.n_w + L.n_b) / batch_params;
      }
    } else {
      pd_layer_profile& u = units[unit_of[m.layer]];
      (m.phase == 0 ? u.fwd_ms : m.phase == 1 ? u.bwd_ms : u.upd_ms) += ms;
    }
  }
  for (pd_layer_profile& u : units) {
    if (st->prof_ops[0]) u.fwd_ms /= st->prof_ops[0];
    if (st->prof_ops[1]) u.bwd_ms /= st->prof_ops[1];
    if (st->prof_ops[2]) u.upd_ms /= st->prof_ops[2];
  }
  memcpy(out, units.data(), units.size() * sizeof(pd_layer_profile));
  return PD_OK;
}

}  // extern "C"

namespace {

// The pipeline drivers join several streams by events; under stream capture that pulls every stage's stream into the
// capture (a wait on an event recorded in a capturing stream forks the waiting stream into it) and nothing joins them
// back to the stream the capture began on, which the capture rules forbid: the capture cannot be ended.  So the
// drivers refuse to run while any of their streams is being captured.
int refuse_capture(pd_stage* const* stages, int n) {
  for (int k = 0; k < n; ++k) {
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    PD_HIP(hipStreamIsCapturing(stages[k]->stream, &cs));
    if (cs == hipStreamCaptureStatusNone && stages[k]->stream_b) PD_HIP(hipStreamIsCapturing(stages[k]->stream_b, &cs));
    if (cs != hipStreamCaptureStatusNone)
      return fail(PD_ESTATE, "the stream of stage object %d is being captured: the pipeline drivers join several streams "
                  "by events and cannot be recorded into a graph (capture pd_forward / pd_backward / pd_update of one "
                  "stage instead)", k);
  }
  return PD_OK;
}

int grow_events(std::vector<hipEvent_t>& v, int n) {
  while ((int)v.size() < n) {
    hipEvent_t e;
    PD_HIP(hipEventCreateWithFlags(&e, hipEventDisableTiming));
    v.push_back(e);
  }
  return PD_OK;
}

}  // namespace

extern "C" {

int pd_pipeline_run(pd_stage* const* stages, int32_t num_stages, int32_t num_minibatches, const void* inputs_dev,
                    const int32_t* labels_dev, float* losses_dev) {
  if (!stages || num_stages < 1) return fail(PD_EINVAL, "no stages");
  if (num_minibatches < 0) return fail(PD_EINVAL, "num_minibatches < 0");
  if (num_minibatches == 0) return PD_OK;
  if (!inputs_dev || !labels_dev) return fail(PD_EINVAL, "inputs_dev / labels_dev is null");
  const int S = num_stages, M = num_minibatches;
  for (int s = 0; s < S; ++s) {
    pd_stage* st = stages[s];
    if (!st) return fail(PD_EINVAL, "stage %d is null", s);
    if (st->stage_index != s || st->num_stages != S) return fail(PD_EINVAL, "stage %d has index %d of %d", s, st->stage_index, st->num_stages);
    if (st->n_replicas > 1) return fail(PD_EINVAL, "stage %d is replicated: its replicas are driven op by op", s);
    if (st->B != stages[0]->B || st->bf16 != stages[0]->bf16) return fail(PD_EINVAL, "stage %d: minibatch/precision differ", s);
    if (s > 0 && (st->lin.front().in != stages[s - 1]->lin.back().out || st->lin.front().rows != stages[s - 1]->lin.back().rows))
      return fail(PD_EINVAL, "stage %d input shape mismatch", s);
    if (st->has_loss != (s == S - 1)) return fail(PD_EINVAL, "only the last stage may (and must) end in the loss");
    if (!st->in_flight.empty() || st->grad_pending) return fail(PD_ESTATE, "stage %d has minibatches in flight", s);
    if (st->last_fwd != stages[0]->last_fwd) return fail(PD_ESTATE, "stages disagree on the next minibatch id");
    if (st->vsync != stages[0]->vsync) return fail(PD_EINVAL, "stage %d: vertical sync must be set on all stages or none", s);
    if (st->vsync && st->latest != stages[0]->latest)
      return fail(PD_ESTATE, "vertical sync: stage %d is at version %d, the input stage at %d", s, st->latest, stages[0]->latest);
  }
  if (refuse_capture(stages, S)) return PD_ESTATE;
  const bool vsync = stages[0]->vsync;
  const int base = stages[0]->last_fwd + 1;
  // Event rings.  Minibatch i of stage s uses ev_f / ev_b / ev_u [i mod R].  R need not grow with the stream: a record
  // of entry i + R is only ever enqueued after every wait on entry i (ev_f[s][i]: F(i, s+1), which the record of
  // F(i + R, s) follows through the update that frees the consumer's input slot, R >= its input-ring depth;
  // ev_b[s][i]: B(i, s-1), R >= 2; ev_u[s][i]: F(i + input-ring depth of s, s-1) and B(i + 2, s+1)).  The checks
  // before each record below assert exactly that, with integers.
  int R = 2;
  for (int s = 0; s < S; ++s) R = std::max(R, stages[s]->in_depth);
  R += 1;
  std::vector<std::vector<pd_op>> ops(S);
  for (int s = 0; s < S; ++s) {
    build_schedule(stages[s]->depth, M, ops[s]);
    for (auto* v : {&stages[s]->ev_f, &stages[s]->ev_b, &stages[s]->ev_u})
      if (grow_events(*v, R)) return PD_EHIP;
  }
  // nF[s], nB[s], nU[s]: forwards, backwards, updates of stage s enqueued so far.  A stage's ops are enqueued in its
  // list order, so "the event of op X(i, s) has been recorded" is i < nX[s].  An op is only enqueued after every event
  // it waits for has been recorded, which makes the host's enqueue order a valid global order.
  std::vector<int> nF(S, 0), nB(S, 0), nU(S, 0);
  std::vector<int> tag(R + 1, -1);  // vertical sync: the version the input stage's forward read, by minibatch mod (R + 1)
  std::vector<size_t> pos(S, 0);
  const size_t in_elems = (size_t)stages[0]->lin.front().rows * stages[0]->lin.front().in * stages[0]->esz;
  size_t remaining = 0;
  for (int s = 0; s < S; ++s) remaining += ops[s].size();
  auto ring_bug = [&](const char* what, int s, int i) {
    return fail(PD_ESTATE, "internal: event ring of %d entries too short for %s of minibatch %d on stage %d", R, what, i, s);
  };
  while (remaining) {
    bool progressed = false;
    for (int s = 0; s < S; ++s) {
      pd_stage* st = stages[s];
      while (pos[s] < ops[s].size()) {
        const pd_op op = ops[s][pos[s]];
        const int i = op.mb_id, mb = base + i, e = i % R;
        if (op.kind == PD_OP_F) {
          int reuse = -1;
          if (s > 0 && i >= nF[s - 1]) break;
          if (s < S - 1) {
            reuse = i - stages[s + 1]->in_depth;  // last minibatch that used the slot this forward writes into
            if (reuse >= 0 && reuse >= nU[s + 1]) break;
          }
          if (s > 0) PD_HIP(hipStreamWaitEvent(st->stream, stages[s - 1]->ev_f[e], 0));
          if (reuse >= 0) PD_HIP(hipStreamWaitEvent(st->stream, stages[s + 1]->ev_u[reuse % R], 0));
          const void* x = s == 0 ? static_cast<const char*>(inputs_dev) + (size_t)i * in_elems : st->in_slot(mb);
          void* y = s < S - 1 ? stages[s + 1]->in_slot(mb) : nullptr;
          const int32_t* lab = s == S - 1 ? labels_dev + (size_t)i * st->lin.back().rows : nullptr;
          float* loss = (s == S - 1 && losses_dev) ? losses_dev + i : nullptr;
          if (vsync && s == 0) tag[i % (R + 1)] = st->latest;
          // zero-copy hand-off: the consumer's input slot stays intact until this stage's backward pass of the
          // minibatch (its next writer is this stage's forward pass `in_depth` minibatches on, which the stage's own
          // list places after that backward pass when in_depth >= depth), so the last layer writes straight into it
          const bool borrow = s < S - 1 && stages[s + 1]->in_depth >= st->depth;
          const int rc = forward_impl(st, mb, vsync ? tag[i % (R + 1)] : -1, x, lab, y, loss, borrow);
          if (rc != PD_OK) return rc;
          if (s < S - 1) {  // (only the next stage waits for it)
            if (i >= R && nF[s + 1] <= i - R) return ring_bug("the forward pass", s, i);
            PD_HIP(hipEventRecord(st->ev_f[e], st->stream));
          }
          ++nF[s];
        } else if (op.kind == PD_OP_B) {
          if (s < S - 1 && i >= nB[s + 1]) break;
          // the gradient slot this backward writes into: the stage before reads it in place (as dL/d(pre-activation)
          // of its last layer) up to and including its update two minibatches back
          if (s > 0 && i >= 2 && i - 2 >= nU[s - 1]) break;
          if (s < S - 1) PD_HIP(hipStreamWaitEvent(st->bstream(), stages[s + 1]->ev_b[e], 0));
          if (s > 0 && i >= 2) PD_HIP(hipStreamWaitEvent(st->bstream(), stages[s - 1]->ev_u[(i - 2) % R], 0));
          const void* dy = s < S - 1 ? st->grad_slot(mb) : nullptr;
          void* dx = s > 0 ? stages[s - 1]->grad_slot(mb) : nullptr;
          // zero-copy hand-off: this stage stores dL/d(input) with the producer's ReLU mask applied (the mask is this
          // stage's own input), and takes what the consumer stored for it as it lies
          const int rc = backward_impl(st, mb, dy, dx, s < S - 1, s > 0 && stages[s - 1]->lin.back().relu);
          if (rc != PD_OK) return rc;
          if (i >= R && ((s > 0 && nB[s - 1] <= i - R) || (s < S - 1 && nB[s + 1] <= i - R + 2)))
            return ring_bug("the backward pass", s, i);
          PD_HIP(hipEventRecord(st->ev_b[e], st->bstream()));
          ++nB[s];
        } else {
          const int rc = pd_update(st);
          if (rc != PD_OK) return rc;
          if (S > 1) {  // (the neighbours wait for it: reuse of this stage's input slot and of its gradient slot)
            if (i >= R && ((s > 0 && nF[s - 1] <= i - R + st->in_depth) || (s < S - 1 && nB[s + 1] <= i - R + 2)))
              return ring_bug("the update", s, i);
            PD_HIP(hipEventRecord(st->ev_u[e], st->stream));
          }
          ++nU[s];
        }
        ++pos[s];
        --remaining;
        progressed = true;
      }
    }
    if (!progressed) return fail(PD_ESTATE, "pipeline cannot make progress (dependency cycle)");
  }
  return PD_OK;
}

// A pipeline whose stages may be replicated (Section 3.3: both the 1F1B policy and the round-robin routing are static,
// so every replica's op list is known in advance).  Replica q of stage s works on minibatches i with i mod r_s == q,
// as its round k = i div r_s; the update of round k of a replicated stage is joint.
int pd_pipeline_run_replicated(pd_stage* const* replicas, const int32_t* replicas_per_stage, int32_t num_stages,
                               int32_t num_minibatches, const void* inputs_dev, const int32_t* labels_dev,
                               float* losses_dev) {
  if (!replicas || !replicas_per_stage || num_stages < 1) return fail(PD_EINVAL, "no stages");
  if (num_minibatches < 0) return fail(PD_EINVAL, "num_minibatches < 0");
  if (num_minibatches == 0) return PD_OK;
  if (!inputs_dev || !labels_dev) return fail(PD_EINVAL, "inputs_dev / labels_dev is null");
  const int S = num_stages, M = num_minibatches;
  std::vector<int> r(S), first(S);  // replicas of stage s: replicas[first[s] .. first[s] + r[s] - 1]
  for (int s = 0, n = 0; s < S; ++s) {
    r[s] = replicas_per_stage[s];
    if (r[s] < 1 || r[s] > pd::kMaxReplicas) return fail(PD_EINVAL, "stage %d: %d replicas", s, r[s]);
    first[s] = n;
    n += r[s];
  }
  auto rep = [&](int s, int q) { return replicas[first[s] + q]; };
  auto rounds = [&](int s, int q) { return q < M ? (M - q + r[s] - 1) / r[s] : 0; };  // minibatches routed to (s, q)
  for (int s = 0; s < S; ++s) {
    pd_stage* p0 = rep(s, 0);
    if (!p0) return fail(PD_EINVAL, "stage %d is null", s);
    if (p0->primary) return fail(PD_EINVAL, "stage %d: its first entry must be the primary", s);
    if ((p0->n_replicas > 1 ? p0->n_replicas : 1) != r[s] || (int)p0->secondaries.size() + 1 != r[s])
      return fail(PD_EINVAL, "stage %d is configured for %d replicas, %zu exist, %d were passed", s, p0->n_replicas,
                  p0->secondaries.size() + 1, r[s]);
    for (int q = 0; q < r[s]; ++q) {
      pd_stage* st = rep(s, q);
      if (!st || (q > 0 && st != p0->secondaries[q - 1])) return fail(PD_EINVAL, "stage %d: replicas must be passed in the order they were created", s);
      if (st->stage_index != s || st->num_stages != S) return fail(PD_EINVAL, "stage %d has index %d of %d", s, st->stage_index, st->num_stages);
      if (st->B != replicas[0]->B || st->bf16 != replicas[0]->bf16) return fail(PD_EINVAL, "stage %d: minibatch/precision differ", s);
      if (st->vsync) return fail(PD_EINVAL, "vertical sync is not available in a pipeline with replicated stages");
      if (!st->in_flight.empty() || st->grad_pending) return fail(PD_ESTATE, "stage %d has minibatches in flight", s);
      if (st->last_fwd != -1 || st->latest != p0->latest) return fail(PD_ESTATE, "stage %d: start from freshly set parameters", s);
      if (st->profiling) return fail(PD_ESTATE, "stage %d: stop the layer profiler first", s);
    }
    if (s > 0 && (p0->lin.front().in != rep(s - 1, 0)->lin.back().out || p0->lin.front().rows != rep(s - 1, 0)->lin.back().rows))
      return fail(PD_EINVAL, "stage %d input shape mismatch", s);
    if (p0->has_loss != (s == S - 1)) return fail(PD_EINVAL, "only the last stage may (and must) end in the loss");
  }
  {
    std::vector<pd_stage*> all;
    for (int s = 0; s < S; ++s)
      for (int q = 0; q < r[s]; ++q) all.push_back(rep(s, q));
    if (refuse_capture(all.data(), (int)all.size())) return PD_ESTATE;
  }
  // Event rings, as in pd_pipeline_run: ev_f / ev_b of a replica by its round modulo R, ev_u of a stage's primary by
  // round modulo R (the joint update).  Between neighbouring stages with different replica counts one round of the
  // one spans up to `ratio` rounds of the other, and a replica only knows about another replica's progress through the
  // joint updates, `depth` rounds back; R covers both, and the checks before each record assert with integers that
  // every wait on the entry's previous occupant has been enqueued.
  int D = 2, ratio = 1;
  for (int s = 0; s < S; ++s) {
    D = std::max(D, rep(s, 0)->in_depth);
    if (s > 0) ratio = std::max(ratio, std::max((r[s] + r[s - 1] - 1) / r[s - 1], (r[s - 1] + r[s] - 1) / r[s]));
  }
  const int R = (2 * D + 6) * ratio;
  // op lists per replica; nF / nB: rounds whose F / B each replica has enqueued; nU: rounds whose joint update a stage
  // has enqueued.  A replica's ops are enqueued in its list order, so "the event of F(k) has been recorded" is k < nF.
  std::vector<std::vector<std::vector<pd_op>>> ops(S);
  std::vector<std::vector<size_t>> pos(S);
  std::vector<std::vector<int>> nF(S), nB(S);
  std::vector<int> nU(S, 0);
  size_t remaining = 0;
  for (int s = 0; s < S; ++s) {
    ops[s].resize(r[s]); pos[s].assign(r[s], 0); nF[s].assign(r[s], 0); nB[s].assign(r[s], 0);
    for (int q = 0; q < r[s]; ++q) {
      pd_stage* st = rep(s, q);
      build_schedule(st->depth, rounds(s, q), ops[s][q]);
      remaining += ops[s][q].size();
      for (auto* v : {&st->ev_f, &st->ev_b, &st->ev_u})
        if (grow_events(*v, R)) return PD_EHIP;
    }
  }
  const size_t in_elems = (size_t)replicas[0]->lin.front().rows * replicas[0]->lin.front().in * replicas[0]->esz;
  auto ring_bug = [&](const char* what, int s, int q, int k) {
    return fail(PD_ESTATE, "internal: event ring of %d entries too short for %s of round %d on stage %d replica %d", R, what, k, s, q);
  };
  // has stage t enqueued the forward (backward) pass of minibatch j?
  auto fwd_done = [&](int t, int j) { return nF[t][j % r[t]] > j / r[t]; };
  auto bwd_done = [&](int t, int j) { return nB[t][j % r[t]] > j / r[t]; };
  // An op is enqueued only after every event it waits for has been recorded (in host order), which makes the host's
  // enqueue order a valid global order.
  while (remaining) {
    bool progressed = false;
    for (int s = 0; s < S; ++s)
      for (int q = 0; q < r[s]; ++q) {
        pd_stage* st = rep(s, q);
        while (pos[s][q] < ops[s][q].size()) {
          const pd_op op = ops[s][q][pos[s][q]];
          const int k = op.mb_id, i = k * r[s] + q;  // round of this replica, minibatch of the stream
          // neighbours of minibatch i: the replica and round that hold it in the stages before and after
          const int qp = s > 0 ? i % r[s - 1] : 0, kp = s > 0 ? i / r[s - 1] : 0;
          const int qn = s < S - 1 ? i % r[s + 1] : 0, kn = s < S - 1 ? i / r[s + 1] : 0;
          if (op.kind == PD_OP_F) {
            int reuse = -1;  // the round whose input last occupied the slot this forward's output goes into
            if (s > 0 && !fwd_done(s - 1, i)) break;
            if (s < S - 1) {
              reuse = kn - rep(s + 1, qn)->in_depth;
              if (reuse >= 0 && reuse >= nU[s + 1]) break;  // its last reader is that round's update
            }
            if (s > 0) PD_HIP(hipStreamWaitEvent(st->stream, rep(s - 1, qp)->ev_f[kp % R], 0));
            if (reuse >= 0) PD_HIP(hipStreamWaitEvent(st->stream, rep(s + 1, 0)->ev_u[reuse % R], 0));
            const void* x = s == 0 ? static_cast<const char*>(inputs_dev) + (size_t)i * in_elems : st->in_slot(k);
            void* y = s < S - 1 ? rep(s + 1, qn)->in_slot(kn) : nullptr;
            const int32_t* lab = s == S - 1 ? labels_dev + (size_t)i * st->lin.back().rows : nullptr;
            float* loss = (s == S - 1 && losses_dev) ? losses_dev + i : nullptr;
            const int rc = pd_forward(st, k, x, lab, y, loss);
            if (rc != PD_OK) return rc;
            if (s < S - 1) {  // (only the next stage waits for it)
              if (k >= R && !fwd_done(s + 1, (k - R) * r[s] + q)) return ring_bug("the forward pass", s, q, k);
              PD_HIP(hipEventRecord(st->ev_f[k % R], st->stream));
            }
            ++nF[s][q];
          } else if (op.kind == PD_OP_B) {
            if (s < S - 1 && !bwd_done(s + 1, i)) break;
            if (s > 0 && kp >= 2 && kp - 2 >= nB[s - 1][qp]) break;  // the gradient slot this backward writes into
            if (s < S - 1) PD_HIP(hipStreamWaitEvent(st->bstream(), rep(s + 1, qn)->ev_b[kn % R], 0));
            if (s > 0 && kp >= 2) PD_HIP(hipStreamWaitEvent(st->bstream(), rep(s - 1, qp)->ev_b[(kp - 2) % R], 0));
            const void* dy = s < S - 1 ? st->grad_slot(k) : nullptr;
            void* dx = s > 0 ? rep(s - 1, qp)->grad_slot(kp) : nullptr;
            const int rc = pd_backward(st, k, dy, dx);
            if (rc != PD_OK) return rc;
            if (k >= R) {  // the entry's previous occupant, round k - R: its two waiters
              const int j = (k - R) * r[s] + q, j2 = (k - R + 2) * r[s] + q;
              if ((s > 0 && !bwd_done(s - 1, j)) || (s < S - 1 && !bwd_done(s + 1, j2))) return ring_bug("the backward pass", s, q, k);
            }
            PD_HIP(hipEventRecord(st->ev_b[k % R], st->bstream()));
            ++nB[s][q];
          } else {
            // joint update of round k: every replica with a minibatch in it must have reached it
            bool ready = true;
            for (int p = 0; p < r[s] && ready; ++p) {
              if (rounds(s, p) <= k) continue;
              const size_t at = pos[s][p];
              ready = at < ops[s][p].size() && ops[s][p][at].kind == PD_OP_U && ops[s][p][at].mb_id == k;
            }
            if (!ready) break;
            const int rc = r[s] > 1 ? pd_update_replicated(replicas + first[s], r[s]) : pd_update(st);
            if (rc != PD_OK) return rc;
            if (s > 0) {  // (only the stage before waits for it)
              if (k >= R) {  // previous occupant: round k - R, waited for by the forwards that refill its input slots
                const int kw = k - R + rep(s, 0)->in_depth;
                for (int j = kw * r[s]; j < (kw + 1) * r[s] && j < M; ++j)
                  if (!fwd_done(s - 1, j)) return ring_bug("the update", s, q, k);
              }
              PD_HIP(hipEventRecord(rep(s, 0)->ev_u[k % R], rep(s, 0)->stream));
            }
            ++nU[s];
            for (int p = 0; p < r[s]; ++p)
              if (p != q && rounds(s, p) > k) {
                ++pos[s][p];
                --remaining;
              }
          }
          ++pos[s][q];
          --remaining;
          progressed = true;
        }
      }
    if (!progressed) return fail(PD_ESTATE, "pipeline cannot make progress (dependency cycle)");
  }
  return PD_OK;
}

int pd_set_big_tile_threshold(int32_t min_tiles) {
  pd::set_conv_wide_min_tiles(2 * min_tiles);  // same rule for the convolutions' 256 x 256 tiles (default 2 x 128)
  return pd::set_big_tile_threshold(min_tiles);
}

int pd_set_big_gemm_waves(int32_t waves) { return pd::set_big_gemm_waves(waves); }
int pd_set_conv_halo(int32_t on) { return pd::set_conv_halo(on); }
int pd_set_recurrence_kernel(int32_t multi_step, uint32_t spin_limit, uint32_t starve) {
  const int old = g_seq_mode;
  g_seq_mode = multi_step ? 1 : 0;
  g_seq_spin_limit = spin_limit ? spin_limit : 4000000u;
  g_seq_starve = starve;
  return old;
}

size_t pd_gemm_workspace_bytes(int32_t M, int32_t N, int32_t K) { return pd::gemm_bf16_workspace_bytes(M, N, K); }

static int check_gemm(const void* a, const void* b, const void* c, int M, int N, int K) {
  if (!a || !b || !c) return fail(PD_EINVAL, "null pointer");
  if (M < 1 || N < 1 || K < 1 || (N % 8) || (K % 8)) return fail(PD_EINVAL, "need M,N,K >= 1 and N,K divisible by 8");
  return PD_OK;
}

int pd_linear_fwd_bf16(void* stream, const void* x, const void* w, const void* b, void* y, int32_t M, int32_t N,
                       int32_t K, int32_t relu, void* workspace_dev, size_t workspace_bytes) {
  if (check_gemm(x, w, y, M, N, K)) return PD_EINVAL;
  PD_HIP(pd::linear_fwd_bf16(static_cast<hipStream_t>(stream), static_cast<const pd::bf16_t*>(x),
                             static_cast<const pd::bf16_t*>(w), static_cast<const pd::bf16_t*>(b),
                             static_cast<pd::bf16_t*>(y), nullptr, M, N, K, relu != 0,
                             static_cast<float*>(workspace_dev), workspace_dev ? workspace_bytes : 0));
  return PD_OK;
}

int pd_linear_dgrad_bf16(void* stream, const void* dz, const void* w, const void* mask, void* dx, int32_t M, int32_t N,
                         int32_t K, void* workspace_dev, size_t workspace_bytes) {
  if (check_gemm(dz, w, dx, M, N, K)) return PD_EINVAL;
  PD_HIP(pd::linear_dgrad_bf16(static_cast<hipStream_t>(stream), static_cast<const pd::bf16_t*>(dz),
                               static_cast<const pd::bf16_t*>(w), static_cast<const pd::bf16_t*>(mask),
                               static_cast<pd::bf16_t*>(dx), M, N, K, static_cast<float*>(workspace_dev),
                               workspace_dev ? workspace_bytes : 0));
  return PD_OK;
}

int pd_linear_wgrad_update_bf16(void* stream, const void* dz, const void* x, float* master_w, float* mom_w,
                                void* ring_out_w, float* master_b, float* mom_b, void* ring_out_b, int32_t M, int32_t N,
                                int32_t K, float lr, float momentum) {
  if (check_gemm(dz, x, master_w, M, N, K)) return PD_EINVAL;
  if (!mom_w || !ring_out_w) return fail(PD_EINVAL, "null pointer");
  if (master_b && (!mom_b || !ring_out_b)) return fail(PD_EINVAL, "bias buffers must be given together");
  pd::WgradBatch batch;
  batch.count = 1; batch.M = M; batch.rule = pd::UpdateRule{lr, momentum, 0.f, 0};
  pd::WgradLayer& W = batch.layer[0];
  W.dz = static_cast<const pd::bf16_t*>(dz); W.x = static_cast<const pd::bf16_t*>(x);
  W.master_w = master_w; W.mom_w = mom_w; W.ring_w = static_cast<pd::bf16_t*>(ring_out_w);
  W.ring_in = nullptr; W.rem_w = nullptr;
  W.master_b = master_b; W.mom_b = mom_b; W.ring_b = static_cast<pd::bf16_t*>(ring_out_b);
  W.M = M; W.N = N; W.K = K; W.tile_end = 0;
  PD_HIP(pd::linear_wgrad_update_bf16(static_cast<hipStream_t>(stream), batch));
  return PD_OK;
}

static int conv_geom(const int32_t* q, pd::ConvGeom& g) {
  if (!q) return fail(PD_EINVAL, "geom is null");
  g = pd::ConvGeom{};
  g.N = q[0]; g.H = q[1]; g.W = q[2]; g.Ci = q[3]; g.Co = q[4]; g.kh = q[5]; g.kw = q[6]; g.stride = q[7];
  g.ph = q[8]; g.pw = q[9];
  if (g.N < 1 || g.H < 1 || g.W < 1 || g.Ci < 1 || g.Co < 1 || g.kh < 1 || g.kw < 1 || g.stride < 1 || g.ph < 0 ||
      g.pw < 0)
    return fail(PD_EINVAL, "bad convolution geometry");
  g.Ho = (g.H + 2 * g.ph - g.kh) / g.stride + 1;
  g.Wo = (g.W + 2 * g.pw - g.kw) / g.stride + 1;
  if (g.Ho < 1 || g.Wo < 1) return fail(PD_EINVAL, "empty convolution output");
  if ((g.Co % 8) || (!pd::conv_is_smallk(g) && (g.Ci % 8)))
    return fail(PD_EINVAL, "channel counts must be divisible by 8 (c_in exempt when kh*kw*c_in <= 32 and c_out <= 64)");
  return PD_OK;
}

static bool plain_product_many_rows(const pd::ConvGeom& g) {
  return g.kh == 1 && g.kw == 1 && g.H == 1 && g.W == 1 && g.N >= kBigRows;
}

// scratch units of (c_out*kh*kw*c_in + c_out) floats that pd_conv_wgrad_update_bf16 uses
static int wgrad_scratch_units(const pd::ConvGeom& g) {
  if (!plain_product_many_rows(g)) return pd::conv_wgrad_split_count(g);
  // one unit for the gradient plus room for the transposed operands
  const size_t unit = ((size_t)g.Co * g.Ci + g.Co) * sizeof(float);
  return 1 + (int)((pd::linear_wgrad_big_scratch_bytes(g.N, g.Co, g.Ci) + unit - 1) / unit);
}

int pd_conv_wgrad_splits(const int32_t* geom, int32_t* splits) {
  pd::ConvGeom g;
  if (conv_geom(geom, g) || !splits) return fail(PD_EINVAL, "bad argument");
  *splits = wgrad_scratch_units(g);
  return PD_OK;
}

int pd_conv_fwd_bf16(void* stream, const void* x, const void* w, const void* b, void* y, const int32_t* geom,
                     int32_t relu) {
  pd::ConvGeom g;
  if (conv_geom(geom, g)) return PD_EINVAL;
  if (!x || !w || !y) return fail(PD_EINVAL, "null pointer");
  const pd::ConvEpilogue ep = {static_cast<const pd::bf16_t*>(b), nullptr, relu ? 1 : 0, static_cast<pd::bf16_t*>(y)};
  PD_HIP(pd::conv_forward_bf16(static_cast<hipStream_t>(stream), static_cast<const pd::bf16_t*>(x),
                               static_cast<const pd::bf16_t*>(w), g, ep));
  return PD_OK;
}

int pd_conv_dgrad_bf16(void* stream, const void* dz, const void* w, const void* mask, void* dx, void* wt_scratch,
                       const int32_t* geom) {
  pd::ConvGeom g;
  if (conv_geom(geom, g)) return PD_EINVAL;
  if (!dz || !w || !dx || !wt_scratch) return fail(PD_EINVAL, "null pointer");
  const pd::ConvEpilogue ep = {nullptr, static_cast<const pd::bf16_t*>(mask), 0, static_cast<pd::bf16_t*>(dx)};
  PD_HIP(pd::conv_dgrad_bf16(static_cast<hipStream_t>(stream), static_cast<const pd::bf16_t*>(dz),
                             static_cast<const pd::bf16_t*>(w), static_cast<pd::bf16_t*>(wt_scratch), g, ep));
  return PD_OK;
}

int pd_conv_wgrad_update_bf16(void* stream, const void* dz, const void* x, float* part_scratch, float* master_w,
                              float* mom_w, void* ring_out_w, float* master_b, float* mom_b, void* ring_out_b,
                              const int32_t* geom, float lr, float momentum) {
  pd::ConvGeom g;
  if (conv_geom(geom, g)) return PD_EINVAL;
  if (!dz || !x || !part_scratch || !master_w || !mom_w || !ring_out_w || !master_b || !mom_b || !ring_out_b)
    return fail(PD_EINVAL, "null pointer");
  int splits = pd::conv_wgrad_split_count(g);
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (plain_product_many_rows(g)) {
    const size_t unit = (size_t)g.Co * g.Ci + g.Co;  // floats per scratch unit; the first holds dw and db
    const size_t extra = (size_t)(wgrad_scratch_units(g) - 1) * unit * sizeof(float);
    PD_HIP(pd::linear_wgrad_update_big_bf16(s, static_cast<const pd::bf16_t*>(dz), static_cast<const pd::bf16_t*>(x),
                                            part_scratch, g.N, g.Co, g.Ci, master_w, mom_w,
                                            static_cast<pd::bf16_t*>(ring_out_w), master_b, mom_b,
                                            static_cast<pd::bf16_t*>(ring_out_b), pd::UpdateRule{lr, momentum, 0.f, 0}, part_scratch + unit,
                                            extra));
    return PD_OK;
  }
  PD_HIP(pd::conv_wgrad_partial_bf16(s, static_cast<const pd::bf16_t*>(dz), static_cast<const pd::bf16_t*>(x),
                                     part_scratch, splits, g));
  PD_HIP(pd::wgrad_reduce_update(s, part_scratch, splits, 0, (size_t)g.Co * g.kh * g.kw * g.Ci, g.Co, master_w, mom_w,
                                 static_cast<pd::bf16_t*>(ring_out_w), master_b, mom_b,
                                 static_cast<pd::bf16_t*>(ring_out_b), pd::UpdateRule{lr, momentum, 0.f, 0}));
  return PD_OK;
}

int pd_maxpool2x2_fwd_bf16(void* stream, const void* x, void* y, int32_t N, int32_t H, int32_t W, int32_t C) {
  return pd_maxpool2x2_fwd_route_bf16(stream, x, y, nullptr, N, H, W, C);
}

int pd_maxpool2x2_fwd_route_bf16(void* stream, const void* x, void* y, uint32_t* route, int32_t N, int32_t H, int32_t W,
                                 int32_t C) {
  if (!x || !y || N < 1 || H < 2 || W < 2 || C < 8 || (C % 8) || (H % 2) || (W % 2))
    return fail(PD_EINVAL, "pooling needs even height/width and channels divisible by 8");
  PD_HIP(pd::maxpool2x2_forward_bf16(static_cast<hipStream_t>(stream), static_cast<const pd::bf16_t*>(x),
                                     static_cast<pd::bf16_t*>(y), route, N, H, W, C));
  return PD_OK;
}

int pd_maxpool2x2_bwd_route_bf16(void* stream, const uint32_t* route, const void* dy, void* dx, int32_t N, int32_t H,
                                 int32_t W, int32_t C, int32_t relu_mask) {
  if (!route || !dy || !dx || N < 1 || H < 2 || W < 2 || C < 8 || (C % 8) || (H % 2) || (W % 2))
    return fail(PD_EINVAL, "pooling needs even height/width and channels divisible by 8");
  PD_HIP(pd::maxpool2x2_backward_routed_bf16(static_cast<hipStream_t>(stream), route,
                                             static_cast<const pd::bf16_t*>(dy), static_cast<pd::bf16_t*>(dx), N, H, W,
                                             C, relu_mask != 0));
  return PD_OK;
}

int pd_maxpool2x2_bwd_bf16(void* stream, const void* x, const void* y, const void* dy, void* dx, int32_t N, int32_t H,
                           int32_t W, int32_t C, int32_t relu_mask) {
  if (!x || !y || !dy || !dx || N < 1 || H < 2 || W < 2 || C < 8 || (C % 8) || (H % 2) || (W % 2))
    return fail(PD_EINVAL, "pooling needs even height/width and channels divisible by 8");
  PD_HIP(pd::maxpool2x2_backward_bf16(static_cast<hipStream_t>(stream), static_cast<const pd::bf16_t*>(x),
                                      static_cast<const pd::bf16_t*>(y), static_cast<const pd::bf16_t*>(dy),
                                      static_cast<pd::bf16_t*>(dx), N, H, W, C, relu_mask != 0));
  return PD_OK;
}

static int pool_geom(const int32_t* q, pd::PoolGeom& g, int is_max) {
  if (!q) return fail(PD_EINVAL, "pgeom is null");
  g = pd::PoolGeom{q[0], q[1], q[2], q[3], q[4], q[5], q[6], 0, 0};
  if (g.N < 1 || g.H < 1 || g.W < 1 || g.C < 8 || (g.C % 8) || g.k < 1 || g.stride < 1 || g.pad < 0 || g.pad >= g.k ||
      g.H + 2 * g.pad < g.k || g.W + 2 * g.pad < g.k || (is_max && g.pad != 0))
    return fail(PD_EINVAL, "pooling needs channels divisible by 8, window/stride >= 1, 0 <= pad < window <= padded "
                "input (max pooling: pad 0)");
  g.Ho = (g.H + 2 * g.pad - g.k) / g.stride + 1;
  g.Wo = (g.W + 2 * g.pad - g.k) / g.stride + 1;
  return PD_OK;
}

int pd_pool2d_fwd_bf16(void* stream, int32_t is_max, const void* x, void* y, const int32_t* pgeom) {
  pd::PoolGeom g;
  if (pool_geom(pgeom, g, is_max)) return PD_EINVAL;
  if (!x || !y) return fail(PD_EINVAL, "null pointer");
  PD_HIP(pd::pool2d_forward_bf16(static_cast<hipStream_t>(stream), is_max != 0, static_cast<const pd::bf16_t*>(x),
                                 static_cast<pd::bf16_t*>(y), nullptr, g));
  return PD_OK;
}

int pd_pool2d_fwd_route_bf16(void* stream, const void* x, void* y, void* route, const int32_t* pgeom) {
  pd::PoolGeom g;
  if (pool_geom(pgeom, g, 1)) return PD_EINVAL;
  if (!x || !y || !route) return fail(PD_EINVAL, "null pointer");
  if (!pd::pool2d_routes(true, g)) return fail(PD_EINVAL, "the routing record covers windows of at most 4 x 4");
  if (reinterpret_cast<uintptr_t>(route) & 7) return fail(PD_EINVAL, "route must be 8-byte aligned");
  PD_HIP(pd::pool2d_forward_bf16(static_cast<hipStream_t>(stream), true, static_cast<const pd::bf16_t*>(x),
                                 static_cast<pd::bf16_t*>(y), route, g));
  return PD_OK;
}

int pd_pool2d_bwd_route_bf16(void* stream, const void* route, const void* dy, void* dx, const int32_t* pgeom,
                             int32_t relu_mask) {
  pd::PoolGeom g;
  if (pool_geom(pgeom, g, 1)) return PD_EINVAL;
  if (!route || !dy || !dx) return fail(PD_EINVAL, "null pointer");
  if (!pd::pool2d_routes(true, g)) return fail(PD_EINVAL, "the routing record covers windows of at most 4 x 4");
  if (reinterpret_cast<uintptr_t>(route) & 7) return fail(PD_EINVAL, "route must be 8-byte aligned");
  PD_HIP(pd::pool2d_backward_routed_bf16(static_cast<hipStream_t>(stream), route, static_cast<const pd::bf16_t*>(dy),
                                         static_cast<pd::bf16_t*>(dx), g, relu_mask != 0));
  return PD_OK;
}

int pd_pool2d_bwd_bf16(void* stream, int32_t is_max, const void* x, const void* y, const void* dy, void* dx,
                       const int32_t* pgeom, int32_t relu_mask) {
  pd::PoolGeom g;
  if (pool_geom(pgeom, g, is_max)) return PD_EINVAL;
  if (!x || !y || !dy || !dx) return fail(PD_EINVAL, "null pointer");
  PD_HIP(pd::pool2d_backward_bf16(static_cast<hipStream_t>(stream), is_max != 0, static_cast<const pd::bf16_t*>(x),
                                  static_cast<const pd::bf16_t*>(y), static_cast<const pd::bf16_t*>(dy),
                                  static_cast<pd::bf16_t*>(dx), g, relu_mask != 0));
  return PD_OK;
}

}  // extern "C"
