/*
 * pd.h -- C ABI of the 1F1B weight-stashed pipeline-stage runtime for MI355X (gfx950).
 *
 * What it is.  One pipeline *stage* of PipeDream (arXiv 1806.03377): a run of
 * consecutive layers that executes forward passes (F), backward passes (B) and
 * weight updates (U) for a stream of minibatches under the one-forward-one-
 * backward policy (Section 3.3), keeping one weight version per in-flight
 * minibatch so that a minibatch's backward pass reads exactly the weights its
 * forward pass read (weight stashing, Section 3.4).  The runtime owns the
 * stage's parameter and intermediate state in device memory and hands work to
 * hand-written HIP kernels (Section 4, stage runtime; the paper's ML worker is
 * replaced by these kernels).  Several stages run on ONE GPU, each on its own
 * HIP stream, exchanging activations and gradients through device buffers.
 *
 * Conventions
 *   - Every function returns a pd_status (0 = PD_OK, negative = error) and never
 *     throws.  pd_last_error() gives a thread-local message for the last failure.
 *     After an error the stage is unchanged unless stated otherwise.
 *   - "dev" pointers are device memory of the current HIP device; "host"
 *     pointers are ordinary host memory.  The caller owns every buffer it passes
 *     (arena, inputs, labels, outputs) and the stream.  The library allocates no
 *     device memory: all stage state lives in the caller's arena, carved once at
 *     pd_stage_create (static allocation, Section 3.5).
 *   - pd_forward / pd_backward / pd_update only ENQUEUE kernels on the stage's
 *     stream and return; they never synchronise, never memset, and are safe to
 *     capture into a HIP graph on that stream (a recorded period of `depth`
 *     steps replays correctly because ring and stash slots repeat with that
 *     period; the host-side counters do not advance on replay).  The pipeline
 *     drivers, which join several streams by events, are not meant to be
 *     captured.  Host-side bookkeeping (versions, stash table)
 *     is advanced at call time, which is valid because a stage's op order is
 *     static.  pd_stage_set_* / pd_stage_get_* synchronise the stream.
 *   - Numbering: stages s = 0..S-1, minibatches i = 0,1,2,..., version v = number
 *     of updates applied so far (v = 0: initial weights).  Ring slot of a version
 *     = v mod depth; stash slot of a minibatch = i mod depth.
 *   - Element types.  PD_F32: activations, gradients, weights all float.
 *     PD_BF16_F32ACC: activations, activation gradients and the ring copies of
 *     the weights are bfloat16 (round-to-nearest-even from fp32); every sum,
 *     bias add, the logits of a stage that ends in the loss, the loss, weight
 *     gradients, master weights and momentum are float.
 *   - Matrices are row-major.  A minibatch activation is [rows][features] with
 *     rows = cfg.minibatch; image activations are [rows][height][width][channels]
 *     (NHWC).  Linear weights are W[out][in], convolution weights W[c_out][kh][kw][c_in].
 *   - Flat parameter vector (pd_stage_set_params and friends): layer by layer in
 *     stage order, each Linear or convolution contributing W then b (out values), an
 *     LSTM W_ih, W_hh, b.
 */
#ifndef PD_H_
#define PD_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pd_stage pd_stage; /* opaque host-side handle */

typedef enum {
  PD_OK = 0,
  PD_EINVAL = -1, /* null pointer, bad shape, bad enum                         */
  PD_ESTATE = -2, /* call violates the 1F1B protocol (see each function)       */
  PD_ENOMEM = -3, /* arena or output array too small                           */
  PD_EHIP = -4    /* a HIP runtime call failed; message holds hipGetErrorString */
} pd_status;

typedef enum { PD_F32 = 0, PD_BF16_F32ACC = 1 } pd_precision;

typedef enum { PD_OP_F = 0, PD_OP_B = 1, PD_OP_U = 2 } pd_op_kind;

/* The update rule of a stage (Section 5.1: SGD with momentum for VGG16 and S2VT, RMSProp for Inception-v3), applied
 * to the fp32 latest weights w with gradient g and ONE fp32 state value per parameter (what pd_stage_get_momentum
 * returns):
 *   PD_OPT_SGD_MOMENTUM  m <- momentum*m + g ;                      w <- w - lr*m
 *   PD_OPT_RMSPROP       v <- momentum*v + (1 - momentum)*g*g ;     w <- w - lr*g / (sqrt(v) + eps)
 *                        (the `momentum` field is the decay of the squared-gradient average) */
typedef enum { PD_OPT_SGD_MOMENTUM = 0, PD_OPT_RMSPROP = 1 } pd_optimizer;

/* One entry of a stage's static schedule (integers only).
 * F, B: `version` = weight version read; U: `version` = weight version produced.
 * `slot` = version mod depth (ring slot read, or written for U). */
typedef struct {
  int32_t kind, mb_id, version, slot;
} pd_op;

typedef enum {
  PD_LINEAR = 0,       /* p[0]=in_features p[1]=out_features p[2]=1: fused ReLU on the output.  After a
                          convolution or pooling layer the input is that layer's output flattened in
                          NHWC order.                                                              */
  PD_SOFTMAX_XENT = 1, /* p[0]=classes; must be the last layer, directly after a PD_LINEAR          */
  PD_CONV2D = 2,       /* cross-correlation with zero padding, NHWC activations, weights
                          W[c_out][kh][kw][c_in], bias per output channel:
                          p[0]=c_in p[1]=c_out p[2]=kh p[3]=kw p[4]=stride p[5]=pad_h p[6]=pad_w
                          p[7]=1: fused ReLU  p[8]=in_h p[9]=in_w.  PD_BF16_F32ACC only; c_out and c_in
                          divisible by 8, except that a layer with kh*kw*c_in <= 32 and c_out <= 64 (the
                          first layer of an image network) may have any c_in.                      */
  PD_MAXPOOL2D = 3,    /* p[0]=window p[1]=stride p[2]=channels p[3]=in_h p[4]=in_w; no padding, channels
                          divisible by 8, output size (in - window)/stride + 1.  The gradient of a window goes
                          to its first maximum in row-major order; where windows overlap, an input position
                          sums what it receives.  (Window 2, stride 2 on even sizes has a faster kernel.)     */
  PD_LSTM = 4,         /* p[0]=input_size p[1]=hidden p[2]=seq_len.  Sequences are TIME-MAJOR:
                          x[seq_len][minibatch][input_size] -> h[seq_len][minibatch][hidden]; gates in the
                          order i, f, g, o = x_t W_ih^T + h_{t-1} W_hh^T + b, c_t = f c_{t-1} + i g,
                          h_t = o tanh(c_t), zero initial state; backward = full back-propagation through
                          time.  Parameters: W_ih[4H][I], W_hh[4H][H], b[4H].  Must be first in its stage
                          or follow another LSTM; layers after it see seq_len*minibatch rows (a Linear
                          acts on every time step; the loss is the mean over all of them, labels
                          [seq_len][minibatch]).  PD_BF16_F32ACC only; sizes divisible by 8.          */
  PD_AVGPOOL2D = 5,    /* p[0]=window p[1]=stride p[2]=pad p[3]=channels p[4]=in_h p[5]=in_w: mean over the
                          window, zero padding counted in the divisor (window*window); pad < window.  A window
                          equal to the input size with stride 1 and pad 0 is global average pooling.          */
  /* A block of parallel branches joined by channel concatenation (Inception-style):
   *   PD_CONCAT_BEGIN, then per branch PD_BRANCH followed by its layers (PD_CONV2D / PD_MAXPOOL2D /
   *   PD_AVGPOOL2D only, at least one), then PD_CONCAT_END.
   * Every branch reads the block's input (the output of the layer before PD_CONCAT_BEGIN, or the stage input);
   * all branches must end with the same height and width; the block's output is [rows][h][w][sum of branch
   * channels], branch 0 first.  Backward: each branch receives its channel slice of dL/d(output); dL/d(input) is
   * the sum of the branches' input gradients (each stored as bf16, added in fp32 in branch order, rounded once).
   * Blocks do not nest; at most 8 branches.  The three markers take no parameters.  PD_BF16_F32ACC only.      */
  PD_CONCAT_BEGIN = 6,
  PD_BRANCH = 7,
  PD_CONCAT_END = 8
} pd_layer_kind;

typedef struct {
  int32_t kind;
  int32_t p[12];
} pd_layer_desc;

typedef struct {
  int32_t stage_index;        /* s, 0-based                                                      */
  int32_t num_stages;         /* S                                                               */
  int32_t noam;               /* NUM_OPT_ACTIVE_MINIBATCHES (Section 3.2); depth = max(1, noam-s) */
  int32_t in_flight_override; /* > 0: use this depth instead (a stage benchmarked alone at
                                 input-stage depth)                                              */
  int32_t minibatch;          /* rows per minibatch                                              */
  int32_t precision;          /* pd_precision                                                    */
  float lr;                   /* learning rate (constant)                                        */
  float momentum;             /* mu in  m <- mu*m + g ; w <- w - lr*m  (Section 5.1: 0.9, 0.01); RMSProp: decay  */
  int32_t n_layers;
  const pd_layer_desc* layers; /* host; copied at create                                          */
  void* stream;               /* hipStream_t, borrowed; all of the stage's kernels run on it      */
  int32_t vertical_sync;      /* != 0: vertical sync (Section 3.4).  The stage keeps as many weight versions as the
                                 INPUT stage (max(1, noam), or in_flight_override) so that a forward pass may ask
                                 for the version its minibatch was tagged with there (pd_forward_versioned);
                                 the in-flight depth is unchanged                                  */
  int32_t optimizer;          /* pd_optimizer; 0 = momentum SGD (the default of a zeroed field)                 */
  float eps;                  /* RMSProp: added to sqrt(v); must be > 0 there, ignored otherwise               */
  int32_t replicas;           /* 0 or 1: an ordinary stage.  2..8: the stage is replicated (Section 3.3); this
                                 object is its primary replica and keeps a gradient buffer of one parameter set;
                                 see pd_stage_create_replica and pd_update_replicated.  Not with vertical_sync  */
  void* stream_backward;      /* NULL: every kernel of the stage runs on `stream`.  Otherwise a second hipStream_t
                                 (borrowed, default priority, not `stream`) on which the kernels of pd_backward run.
                                 In the 1F1B order F(k + depth) is followed by B(k + 1), and the two do not depend
                                 on each other: with a stream of its own the backward pass runs next to that forward
                                 pass instead of behind it.  The library orders what it must with events: what a
                                 backward pass leaves for pd_update exists twice in this mode and consecutive passes
                                 alternate, so a backward pass starts after its minibatch's forward pass and after the
                                 update BEFORE the last one (the reader of the buffers it overwrites); pd_update
                                 starts after the backward pass.  The arena grows by those buffers and a workspace.  Results are the
                                 same bit for bit.  What pd_backward reads from the caller (dy_dev) must be complete,
                                 or ordered by the caller on stream_backward, when it is called; what it writes
                                 (dx_dev) is complete on stream_backward, and on `stream` after the following
                                 pd_update.  Such a stage cannot be captured into a HIP graph, profiled per layer
                                 (pd_stage_profile) or replicated.                                              */
} pd_stage_config;

/* --- schedule (pure host, no GPU touched) -------------------------------------------------
 * The static per-stage op list of the 1F1B policy (Section 3.3): `depth` forwards at
 * start-up (depth = max(1, noam - stage_index): the input stage admits NOAM, the output stage
 * one, Sections 3.3 and 3.5; fewer if the stream is shorter), then alternately the backward of
 * the oldest in-flight minibatch -- followed at once by its update -- and the next forward;
 * remaining backwards drain in order at the end.  Versions follow weight stashing (Section
 * 3.4): F reads the latest version, B the version its F read, U produces latest+1.
 * Writes up to `cap` ops to `out` (host) and the full count (3 * num_minibatches) to *n_out.
 * PD_ENOMEM if cap is too small (n_out still set); PD_EINVAL on bad arguments. */
int pd_schedule_1f1b(int32_t num_stages, int32_t noam, int32_t num_minibatches, int32_t stage_index,
                     pd_op* out, size_t cap, size_t* n_out);
/* The list of the same stage under vertical sync (Section 3.4): same op order; F and B carry the version the
 * INPUT stage's forward of that minibatch read, and slot = version mod (depth of the input stage). */
int pd_schedule_1f1b_vertical_sync(int32_t num_stages, int32_t noam, int32_t num_minibatches, int32_t stage_index,
                                   pd_op* out, size_t cap, size_t* n_out);
/* Same list for an explicitly given in-flight depth (>= 1). */
int pd_schedule_1f1b_depth(int32_t depth, int32_t num_minibatches, pd_op* out, size_t cap, size_t* n_out);

/* --- stage life cycle (Sections 3.5 and 4: static allocation at initialisation) -----------
 * pd_stage_query_bytes: bytes of device arena the configuration needs (weight-version ring,
 * fp32 master weights and momentum, in bf16 mode 16-bit remainders of the master weights,
 * activation stash for `depth` minibatches, input ring, gradient and split-K workspaces).
 * pd_stage_create: carves `device_arena` (256-byte aligned, >= query bytes, owned by the
 * caller, must outlive the stage; contents need not be initialised).  Parameters start
 * undefined until pd_stage_set_params; momentum starts at zero.  PD_ENOMEM if too small. */
int pd_stage_query_bytes(const pd_stage_config* cfg, size_t* device_bytes);
int pd_stage_create(const pd_stage_config* cfg, void* device_arena, size_t arena_bytes, pd_stage** out);
int pd_stage_destroy(pd_stage* st);

/* --- replicated stage (Section 3.3: deterministic round-robin over the replicas of a stage; Section 4, "Data
 * Parallelism": the replicas' gradients are aggregated before new parameters are handed out) -----------------------
 * On one GPU the replicas of a stage are pd_stage objects that SHARE one parameter state (version ring, fp32 latest
 * weights, optimiser state: the primary's, created by pd_stage_create with cfg.replicas = r >= 2) and each own a
 * stash, scratch, a gradient buffer and a stream.  What the paper leaves open is read as follows: minibatch i goes to
 * replica i mod r as that replica's round i div r (pd_replica_route); every replica follows the stage's ordinary 1F1B
 * list over its rounds, with `mb_id` = round in pd_forward / pd_backward; the gradients of one round are SUMMED in
 * replica order and applied in one step (pd_update_replicated), after the backward passes of the round on all
 * replicas and before any replica's next forward pass, so weight version = rounds completed; replicas without a
 * minibatch in the last round of a stream only receive the new version.
 *
 * pd_replica_route: pure host arithmetic; PD_EINVAL if mb_id < 0 or n_replicas < 1.
 * pd_stage_replica_query_bytes: arena bytes of one FURTHER replica (no parameter state) for the primary's config.
 * pd_stage_create_replica: a further replica of `primary` on `stream` (borrowed; may equal the primary's), carved
 *   from `device_arena` (256-byte aligned, caller-owned, outlives the replica).  Created in replica order 1..r-1,
 *   with nothing in flight on the primary.  Calls that write the parameter state (pd_stage_set_params,
 *   pd_stage_set_momentum, pd_stage_overwrite_latest, pd_stage_checkpoint_load) are made on the primary only
 *   (PD_ESTATE otherwise) and reset/advance every replica with it; reads work on any replica.  Destroy the further
 *   replicas before the primary (PD_ESTATE otherwise).
 * pd_update_replicated: `replicas` = host array {primary, replica 1, ..., replica r-1}.  Every replica that has a
 *   pending gradient (pd_backward since the last update) contributes; at least one must (PD_ESTATE otherwise).  Its
 *   gradient kernels run on that replica's stream; the summed step runs on the primary's stream once every replica's
 *   stream has reached this call, and every replica's stream waits for it, so no host synchronisation is needed
 *   between the call and the next pd_forward.  pd_update on a replicated stage returns PD_ESTATE; pd_pipeline_run
 *   does not take replicated stages (PD_EINVAL): pd_pipeline_run_replicated does. */
int pd_replica_route(int32_t mb_id, int32_t n_replicas, int32_t* replica, int32_t* round);
int pd_stage_replica_query_bytes(const pd_stage_config* cfg, size_t* device_bytes);
int pd_stage_create_replica(pd_stage* primary, void* stream, void* device_arena, size_t arena_bytes, pd_stage** out);
int pd_update_replicated(pd_stage* const* replicas, int32_t n_replicas);

/* Number of parameters (length of the flat vector), in-flight depth, input-ring depth. */
int pd_stage_num_params(const pd_stage* st, size_t* n);
int pd_stage_depth(const pd_stage* st, int32_t* depth, int32_t* input_ring_depth);
/* Number of weight versions the stage keeps (= depth, or the input stage's depth under vertical sync);
 * ring slot of a version = version mod this. */
int pd_stage_ring_depth(const pd_stage* st, int32_t* ring_depth);

/* Resets the stage to version 0 with these weights (host, fp32, flat layout above), zero
 * momentum, nothing in flight.  In bf16 mode ring slot 0 = round-to-nearest-even of them. */
int pd_stage_set_params(pd_stage* st, const float* host_params, size_t n);
/* Weights of `version` (-1 = latest) as fp32 into host_out.  Latest: the fp32 master.  (bf16 mode, unreplicated
 * stage: the master weights of Linear and LSTM layers with minibatch-sized row counts are held as the latest bf16 ring
 * copy plus the low 16 bits of their fp32 pattern, which is exact for every value but one kind: a value whose low
 * half is exactly 0x8000 and whose upper half is even -- a tie that rounds down -- is held, and returned, one fp32 unit
 * in the last place lower.  This applies to what set_params / overwrite_latest store and to what an update produces.
 * NaNs are not preserved.)  An older
 * version must still be in the ring (version > latest - depth), else PD_ESTATE; in bf16 mode
 * an older version is its bf16 ring copy widened to float.  `ring_copy` != 0 forces the ring
 * copy also for the latest version. */
int pd_stage_get_params(pd_stage* st, int32_t version, int32_t ring_copy, float* host_out, size_t n);
/* Momentum buffer (fp32, flat layout).  set requires nothing in flight. */
int pd_stage_set_momentum(pd_stage* st, const float* host_mom, size_t n);
/* Learning rate of the following updates (Section 5.1: Inception-v3's rate is decayed per epoch; the schedule itself is
 * the caller's).  Host-side only: updates already enqueued keep the rate they were launched with.  On the primary of a
 * replicated stage (PD_ESTATE on a further replica).  PD_EINVAL unless finite and >= 0. */
int pd_stage_set_lr(pd_stage* st, float lr);
int pd_stage_get_momentum(pd_stage* st, float* host_out, size_t n);

/* Per-stage checkpoint (Section 4, "Checkpointing": every stage dumps its own parameters when it has done the
 * backward pass -- here: the update -- of an epoch's last minibatch; no coordination between stages).
 * save: writes the LATEST fp32 weights, the momentum and the version id to `path` (host file; synchronises the
 *       stream).  Minibatches may be in flight; PD_ESTATE between pd_backward and pd_update.
 * load: restores them into a stage of the same shape and precision: nothing in flight, version id as saved (the
 *       weights go into that version's ring slot, in bf16 mode rounded from the fp32 values), any next minibatch id.
 *       PD_EINVAL for a missing, truncated or corrupt file (header, size and checksum are verified) or a mismatch.
 * info: header of a checkpoint file (verifies it as load does); pure host, no GPU touched.
 * File layout: "PDCKPT1\0", u32 precision, u32 0, u64 n_params, i64 version, u64 checksum, n_params floats of
 * weights, n_params floats of momentum (flat parameter layout, little-endian); checksum over both arrays taken
 * 8 bytes at a time, h = (h ^ word) * 0x100000001b3 from h = 0xcbf29ce484222325 (an odd tail word is zero-extended
 * per array). */
int pd_stage_checkpoint_save(pd_stage* st, const char* path);
int pd_stage_checkpoint_load(pd_stage* st, const char* path);
int pd_checkpoint_info(const char* path, size_t* n_params, int32_t* latest, int32_t* precision);

/* Waits for everything the stage has enqueued (both of its streams) and reports what only the device can know: an
 * LSTM layer whose time steps ran in one launch has workgroups that wait for each other with a bounded number of
 * polls; if one of them gave up, this call (like every other call that synchronises: pd_stage_get_params, ...)
 * returns PD_ESTATE once and clears the condition.  The stage's state after that minibatch is not valid. */
int pd_stage_check(pd_stage* st);

/* Version bookkeeping: mb_id = -1 -> latest version; otherwise the version stashed for that
 * in-flight minibatch (PD_ESTATE if it is not in flight). */
int pd_stage_version(const pd_stage* st, int32_t mb_id, int32_t* version);
/* The ops executed so far, in order (same encoding as pd_schedule_1f1b).  The stage keeps the most recent 65536
 * ops (pd_stage_set_trace_limit in pd_debug.h changes that or switches the record off); older ones are dropped,
 * so a long-running stage holds a bounded record. */
int pd_stage_trace(const pd_stage* st, pd_op* out, size_t cap, size_t* n_out);

/* Device address of the stage's own input slot for minibatch mb_id ([minibatch][in_features],
 * element type per precision).  A producer (the previous stage's pd_forward, via y_dev) may
 * write the activation straight there; pd_forward then takes it without a copy.  The input
 * ring has depth+1 slots for stage_index > 0 (the producer may run one forward ahead of what
 * this stage has released) and depth slots for stage 0; slot = mb_id mod that depth. */
int pd_stage_input_slot(pd_stage* st, int32_t mb_id, void** dev_ptr);
/* Device address of the buffer that receives dL/d(output) for the backward pass of mb_id
 * ([minibatch][out_features]); two slots, slot = mb_id mod 2. */
int pd_stage_grad_slot(pd_stage* st, int32_t mb_id, void** dev_ptr);

/* --- the step (Sections 3.3, 3.4, 4) -------------------------------------------------------
 * pd_forward: F for minibatch mb_id.  Reads the LATEST weight version and records it in the
 * stash for this minibatch (weight stashing, Section 3.4); runs the layers; keeps each layer's
 * input/output for the backward pass (Section 4, intermediate state).
 *   x_dev      [minibatch][in]: the input.  If it is not the stage's own input slot it is
 *              copied there (on the stream), so the caller may reuse x_dev after that copy.
 *   labels_dev int32[minibatch], required iff the stage ends in PD_SOFTMAX_XENT; then the loss
 *              (mean over rows of -log softmax[label], Section 3.1: the output stage computes
 *              the loss) goes to loss_dev (one float, may be NULL) and dL/dlogits is stashed.
 *   y_dev      [minibatch][out] output of the last non-loss layer, may be NULL.  On a stage
 *              that ends in the loss these are the logits and are float in both precisions.
 * PD_ESTATE if `depth` minibatches are already in flight or mb_id is not the previous
 * forward's id + 1 (first call after set_params: any id >= 0).
 *
 * pd_backward: B for minibatch mb_id, which must be the OLDEST in flight (PD_ESTATE otherwise).
 * Uses the weight version stashed at its forward.  dy_dev [minibatch][out] = dL/d(output),
 * NULL iff the stage ends in the loss.  dx_dev [minibatch][in] receives dL/d(input), NULL to
 * skip it (input stage).  Leaves the weight gradient pending (Linear: held in factored form, per layer
 * dL/d(pre-activation) and the stashed layer input; convolution: fp32 partial sums over pixel ranges)
 * and releases the minibatch's stash slot.
 *
 * pd_update: U.  Consumes the pending gradient: per Linear, dW = dZ^T X and db = colsum(dZ)
 * are formed tile by tile and, in the same kernel, m <- mu*m + g, w <- w - lr*m is applied to
 * the LATEST weights (Section 4, parameter state) and the result stored as version latest+1
 * in ring slot (latest+1) mod depth; per convolution the partial sums are added in a fixed order
 * and the same step applied.  PD_ESTATE without a pending gradient. */
int pd_forward(pd_stage* st, int32_t mb_id, const void* x_dev, const int32_t* labels_dev, void* y_dev,
               float* loss_dev);
/* pd_forward with the weight version given by the caller (vertical sync, Section 3.4: the version travels with the
 * minibatch from the input stage).  version = -1 means the latest (identical to pd_forward); otherwise it must
 * still be in the ring (latest - ring depth < version <= latest), else PD_ESTATE.  The minibatch's backward pass
 * uses the same version, as always.  pd_pipeline_run does this by itself for stages created with vertical_sync. */
int pd_forward_versioned(pd_stage* st, int32_t mb_id, int32_t version, const void* x_dev, const int32_t* labels_dev,
                         void* y_dev, float* loss_dev);
int pd_backward(pd_stage* st, int32_t mb_id, const void* dy_dev, void* dx_dev);
int pd_update(pd_stage* st);

/* --- all stages of a pipeline on one GPU (Section 3.1 / 3.3) -------------------------------
 * Runs num_minibatches through stages[0..num_stages-1] (stage k must have stage_index k, all
 * the same minibatch and precision, matching widths, the last ending in PD_SOFTMAX_XENT).  Each
 * stage follows its own pd_schedule_1f1b list on its own stream; F(i,s) waits (event) for
 * F(i,s-1), B(i,s) for B(i,s+1); every reuse of an inter-stage slot waits for its last reader.
 * Hand-off without copies: the last layer of stage s writes its output straight into the input slot
 * of stage s+1 (and keeps no other copy: that slot stays intact until stage s has run the minibatch's
 * backward pass); stage s+1 stores dL/d(its input) into the gradient slot of stage s with the ReLU mask
 * of stage s's last layer already applied (the mask is stage s+1's own input), and stage s uses it where
 * it lies, up to and including its update.  (pd_forward / pd_backward called directly copy instead:
 * they cannot know how long the caller's buffers stay intact.)  inputs_dev [num_minibatches][minibatch][in0]; labels_dev int32 [num_minibatches]
 * [minibatch]; losses_dev float[num_minibatches] (may be NULL).  Enqueues everything and
 * returns; the caller synchronises the streams.  Stages must have nothing in flight; minibatch
 * ids continue from each stage's last forward (or 0). */
int pd_pipeline_run(pd_stage* const* stages, int32_t num_stages, int32_t num_minibatches,
                    const void* inputs_dev, const int32_t* labels_dev, float* losses_dev);
/* The same for a pipeline whose stages may be replicated (Section 3.3: the 1F1B policy and the round-robin routing are
 * both static, so every replica's op list is known in advance).  `replicas` lists all stage objects stage by stage,
 * each stage's primary first and its further replicas in creation order; replicas_per_stage[s] = r_s (1 for a stage
 * that is not replicated).  Minibatch i is round i div r_s of replica i mod r_s in stage s; each replica follows the
 * stage's 1F1B list over its rounds on its own stream; the update of a round is joint (pd_update_replicated) and waits
 * for the round's backward passes on every replica that has a minibatch in it.  Hand-off as in pd_pipeline_run, into
 * the input / gradient slot of the replica that holds the minibatch in the neighbouring stage.  All stages must be
 * freshly initialised (nothing run since pd_stage_set_params); no vertical sync.  inputs_dev, labels_dev and losses_dev
 * are indexed by minibatch i as above. */
int pd_pipeline_run_replicated(pd_stage* const* replicas, const int32_t* replicas_per_stage, int32_t num_stages,
                               int32_t num_minibatches, const void* inputs_dev, const int32_t* labels_dev,
                               float* losses_dev);

/* --- profiling and partitioning (Section 3.2) -----------------------------------------------
 * The step before the pipeline runs: measure every layer on the device, then choose the stages.
 *
 * pd_stage_profile: enable != 0 clears earlier records and makes every pd_forward / pd_backward / pd_update
 * of this stage drop a HIP event after each layer's kernels; 0 stops recording.  pd_stage_profile_read waits
 * for the stream and reports one entry per profile UNIT in stage order: a compute layer outside any block of
 * branches, or a whole block (a pipeline can only be cut between units).  first_layer / last_layer use the
 * compute-layer numbering of pd_stage_debug_read.  fwd_ms, bwd_ms, upd_ms = mean time per recorded F, B, U
 * (the time of a launch that updates several Linear layers at once is shared out by parameter count); the
 * paper's T_l is their sum (its backward pass includes the weight gradient, which here is formed in
 * pd_update).  act_bytes = a_l: bytes of the unit's output for one minibatch (also the size of the gradient
 * that comes back); param_bytes = |w_l| as fp32.  Writes up to cap entries, the count to *n_out
 * (PD_ENOMEM if cap is too small, n_out still set). */
typedef struct {
  int32_t first_layer, last_layer;
  double fwd_ms, bwd_ms, upd_ms;
  double act_bytes, param_bytes;
} pd_layer_profile;
int pd_stage_profile(pd_stage* st, int32_t enable);
int pd_stage_profile_read(pd_stage* st, pd_layer_profile* out, size_t cap, size_t* n_out);

/* pd_partition (pure host, no GPU touched): the dynamic program of Section 3.2 over n_layers profile units and
 * n_machines workers.  t_layer[l] = T_l (any time unit), act_bytes[l] = a_l, param_bytes[l] = |w_l| (host
 * arrays of n_layers doubles, all >= 0); bandwidth in bytes per that time unit, > 0.  A stage holding layers
 * i..j replicated over m workers costs max(sum T_l, sum W_l^m) / m with W_l^m = 4 (m-1) |w_l| / (m bandwidth);
 * a boundary after layer i costs 2 a_i / bandwidth; the pipeline's cost is its slowest stage or boundary, all
 * n_machines workers are used.  Outputs (each may be NULL except stages_out when cap > 0): *slowest_out = the
 * optimum A(N, M); stages_out[k] = {first_layer, last_layer (0-based, inclusive), replicas} in pipeline order,
 * *n_stages_out their count; *noam_out = ceil(n_machines / replicas of the input stage), the number of
 * minibatches to keep in flight.  Among partitions of equal cost the one found first wins (split points and
 * replica counts of the last stage in increasing order).  PD_EINVAL on bad arguments; PD_ENOMEM if cap is too
 * small (counts still set). */
typedef struct {
  int32_t first_layer, last_layer, replicas;
} pd_stage_assign;
int pd_partition(int32_t n_layers, int32_t n_machines, const double* t_layer, const double* act_bytes,
                 const double* param_bytes, double bandwidth, double* slowest_out, pd_stage_assign* stages_out,
                 size_t cap, size_t* n_stages_out, int32_t* noam_out);

/* --- stand-alone kernels of the step, for measurement at other shapes ----------------------
 * The same GEMM kernels the stage uses, callable on caller buffers (bf16 data, fp32
 * accumulate), so that MFMA utilisation can be measured at any minibatch size.
 *   fwd   : y[M][N]  = act(x[M][K] * w[N][K]^T + b[N])       (relu != 0: max(.,0))
 *   dgrad : dx[M][K] = (dz[M][N] * w[N][K]) .* (mask[M][K] > 0 if mask != NULL)
 *   wgrad_update: g = dz[M][N]^T x[M][K] (+ column sums for the bias); m <- mu*m+g;
 *           master <- master - lr*m; ring_out <- bf16(master)
 * workspace_dev: split-K scratch of at least pd_gemm_workspace_bytes(M,N,K) bytes (fwd, dgrad); NULL
 * disables split-K.
 * stream: hipStream_t.  All pointers device. */
size_t pd_gemm_workspace_bytes(int32_t M, int32_t N, int32_t K);
int pd_linear_fwd_bf16(void* stream, const void* x, const void* w, const void* b, void* y, int32_t M, int32_t N,
                       int32_t K, int32_t relu, void* workspace_dev, size_t workspace_bytes);
/* pd_linear_fwd_bf16 for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same product, same kernels, same result as
 * pd_linear_fwd_bf16 given a workspace of 32 * M * N * 4 bytes; the split-K partial sums go into a device array that
 * is part of the library image (pd_linear_fwd_bf16_static_max_bytes() = 32 MiB on every GPU the process uses, held
 * until the process ends).  Allocates nothing, frees nothing, synchronises nothing; x, w, b, y are the caller's.
 * Runs on the CURRENT device, which must be the stream's.  PD_ENOMEM if 32 * M * N * 4 exceeds the array (M * N >
 * 262144, e.g. more than 64 rows at 4096 features): use pd_linear_fwd_bf16 there.  All calls on one GPU share the
 * array, which keeps the previous call's contents (no call depends on them): calls on different streams of one GPU
 * must not overlap in time, calls on one stream are ordered and safe. */
size_t pd_linear_fwd_bf16_static_max_bytes(void);
int pd_linear_fwd_bf16_static(void* stream, const void* x, const void* w, const void* b, void* y, int32_t M, int32_t N,
                              int32_t K, int32_t relu);
int pd_linear_dgrad_bf16(void* stream, const void* dz, const void* w, const void* mask, void* dx, int32_t M,
                         int32_t N, int32_t K, void* workspace_dev, size_t workspace_bytes);
int pd_linear_wgrad_update_bf16(void* stream, const void* dz, const void* x, float* master_w, float* mom_w,
                                void* ring_out_w, float* master_b, float* mom_b, void* ring_out_b, int32_t M,
                                int32_t N, int32_t K, float lr, float momentum);

/* Convolution and pooling kernels on caller buffers (bf16 NHWC data, fp32 accumulate; all pointers device).
 * geom = {N, H, W, c_in, c_out, kh, kw, stride, pad_h, pad_w} (10 ints, host); output size
 * Ho = (H + 2 pad_h - kh)/stride + 1, Wo likewise.  Shape rules as for PD_CONV2D / PD_MAXPOOL2D.
 *   conv_fwd  : y[N][Ho][Wo][c_out] = act(conv(x, w) + b)                      (b may be NULL)
 *   conv_dgrad: dx[N][H][W][c_in]   = convT(dz, w) .* (mask > 0 if mask)       any stride;
 *               wt_scratch: c_out*kh*kw*c_in bf16 elements of scratch
 *   conv_wgrad_update: g = dL/dw from dz and x (and column sums for the bias), partial sums over
 *               pixel ranges in part_scratch, added in a fixed order; part_scratch must hold
 *               pd_conv_wgrad_splits(geom) units of (c_out*kh*kw*c_in + c_out) floats; then m <- mu*m + g;
 *               master <- master - lr*m; ring_out <- bf16(master)
 *   maxpool2x2_fwd / _bwd: 2x2 stride-2 max pooling of x[N][H][W][C]; backward routes dy to the first
 *               maximum of each window and, if relu_mask != 0, zeroes positions where x <= 0
 *   maxpool2x2_fwd_route / _bwd_route: the same pair with the routing recorded by the forward pass: route (device,
 *               written by _fwd_route, read by _bwd_route; may be NULL in _fwd_route) holds
 *               N*(H/2)*(W/2)*(C/8) 32-bit words, four bits per output element; _bwd_route gives exactly what _bwd
 *               gives without reading x or y (this is what a stage's backward pass runs)
 *   pool2d_fwd / _bwd: pooling with any window, stride and padding (is_max != 0: max, padding never wins, pad
 *               must be 0 < window; else average with divisor window*window); pgeom = {N, H, W, C, window,
 *               stride, pad} (7 ints, host); backward as for PD_MAXPOOL2D / PD_AVGPOOL2D
 *   pool2d_fwd_route / _bwd_route: max pooling with a window of at most 4 x 4 and the routing recorded by the forward
 *               pass: route (device, 8-byte aligned, written by _fwd_route, read by _bwd_route) holds one byte per
 *               output element, N*Ho*Wo*C bytes; _bwd_route gives exactly what _bwd gives without reading x or y
 *               (this is what a stage's backward pass runs for such a layer); other windows: PD_EINVAL */
int pd_conv_wgrad_splits(const int32_t* geom, int32_t* splits);
int pd_conv_fwd_bf16(void* stream, const void* x, const void* w, const void* b, void* y, const int32_t* geom,
                     int32_t relu);
int pd_conv_dgrad_bf16(void* stream, const void* dz, const void* w, const void* mask, void* dx, void* wt_scratch,
                       const int32_t* geom);
int pd_conv_wgrad_update_bf16(void* stream, const void* dz, const void* x, float* part_scratch, float* master_w,
                              float* mom_w, void* ring_out_w, float* master_b, float* mom_b, void* ring_out_b,
                              const int32_t* geom, float lr, float momentum);
int pd_maxpool2x2_fwd_bf16(void* stream, const void* x, void* y, int32_t N, int32_t H, int32_t W, int32_t C);
int pd_maxpool2x2_bwd_bf16(void* stream, const void* x, const void* y, const void* dy, void* dx, int32_t N, int32_t H,
                           int32_t W, int32_t C, int32_t relu_mask);
int pd_maxpool2x2_fwd_route_bf16(void* stream, const void* x, void* y, uint32_t* route, int32_t N, int32_t H, int32_t W,
                                 int32_t C);
int pd_maxpool2x2_bwd_route_bf16(void* stream, const uint32_t* route, const void* dy, void* dx, int32_t N, int32_t H,
                                 int32_t W, int32_t C, int32_t relu_mask);
int pd_pool2d_fwd_bf16(void* stream, int32_t is_max, const void* x, void* y, const int32_t* pgeom);
int pd_pool2d_bwd_bf16(void* stream, int32_t is_max, const void* x, const void* y, const void* dy, void* dx,
                       const int32_t* pgeom, int32_t relu_mask);
int pd_pool2d_fwd_route_bf16(void* stream, const void* x, void* y, void* route, const int32_t* pgeom);
int pd_pool2d_bwd_route_bf16(void* stream, const void* route, const void* dy, void* dx, const int32_t* pgeom,
                             int32_t relu_mask);

const char* pd_last_error(void); /* thread-local, static storage, never NULL */

#ifdef __cplusplus
}
#endif
#endif /* PD_H_ */
