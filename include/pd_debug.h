/*
 * pd_debug.h -- test hooks and tuning knobs of the stage runtime declared in pd.h.
 *
 * Nothing here is part of the training step (Sections 3.3, 3.4, 4 of PipeDream, arXiv 1806.03377): these calls let a
 * test read or overwrite what a stage holds, so that every op can be compared on identical state, and let a
 * measurement force a kernel choice.  They synchronise the stage's stream unless stated otherwise and follow the
 * conventions of pd.h (status codes, pd_last_error, host / device pointers).
 */
#ifndef PD_DEBUG_H_
#define PD_DEBUG_H_

#include "pd.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Overwrites the LATEST version in place: fp32 master <- host_params, its ring slot <- their bf16
 * rounding (bf16 mode), momentum <- host_mom (either may be NULL to leave it).  Version ids, the
 * stash and in-flight minibatches are untouched, so a driver can re-synchronise a running stage
 * with externally computed state (checkpoint restore mid-stream, teacher-forced tests).
 * PD_ESTATE while a gradient is pending (between pd_backward and pd_update). */
int pd_stage_overwrite_latest(pd_stage* st, const float* host_params, const float* host_mom, size_t n);

/* Test/debug aid: copies one of the stage's intermediate tensors to the host as fp32
 * (synchronises the stream).  what = 0: stored output of compute layer number `layer` (0-based, the
 * loss not counted; inside a block of branches the branch layers count in description order and
 * PD_CONCAT_END counts as one more layer whose output is the concatenation; the markers PD_CONCAT_BEGIN
 * and PD_BRANCH do not count) for in-flight minibatch mb_id, [minibatch][out]; 1: the stage's input
 * slot for mb_id, [minibatch][in]; 2: the output-gradient slot for mb_id, [minibatch][out_last];
 * 3: dL/d(pre-activation) of layer `layer` left by the last pd_backward, [minibatch][out] (Linear layers
 * only: convolution and pooling layers do not keep theirs);
 * 4: the stashed dL/dlogits of in-flight minibatch mb_id (loss stages).  n must equal the tensor's
 * element count.  No state check is made on mb_id beyond >= 0: the caller reads what the slot holds. */
int pd_stage_debug_read(pd_stage* st, int32_t what, int32_t mb_id, int32_t layer, float* host_out, size_t n);
/* Test/debug aid, the reverse direction: overwrites a stored tensor of in-flight minibatch mb_id with host values
 * (fp32, rounded to bfloat16 where the tensor is bfloat16; synchronises the stream).  what = 0: the stored output
 * of compute layer `layer` (not an LSTM); 1: the stage's input slot.  Lets a test drive the backward pass of a deep
 * stage on exactly the activations (and therefore the ReLU and max-pooling decisions) of a reference run.  If the
 * minibatch's forward pass has run, a max-pooling layer that reads the overwritten tensor pools it again, so that the
 * routing it recorded in the forward pass (and its stored output) belong to the new values. */
int pd_stage_debug_write(pd_stage* st, int32_t what, int32_t mb_id, int32_t layer, const float* host_in, size_t n);

/* Tuning knob (process-wide, not thread-safe): forward and dgrad products whose output has at least `min_tiles`
 * tiles of 256 x 256 run on the compute-bound large-tile kernels, smaller ones on the split-K kernels built for
 * minibatch-sized row counts.  Default 128.  The same knob (times two) decides from how many 256 x 256 output tiles
 * a convolution with >= 256 output channels uses its wide-tile kernel.  Returns the previous value; min_tiles < 1 only queries.  Set it
 * before pd_gemm_workspace_bytes / pd_stage_query_bytes: the workspace size depends on it. */
int pd_set_big_tile_threshold(int32_t min_tiles);
/* Tuning knob (process-wide, not thread-safe): variant of the large-tile forward product.  0: chosen by the
 * reduction length (the default); 4: four waves of 128 x 128 outputs (one per SIMD); 8: eight waves of 128 x 64;
 * 104 / 108: the same with 64-byte instead of 128-byte tile rows in LDS (32 instead of 64 reduction elements per
 * stage).  Returns the previous value in the same encoding; any other argument only queries. */
int pd_set_big_gemm_waves(int32_t waves);

/* Tuning knob (process-wide, not thread-safe): 1 (default) lets 3 x 3, stride-1, pad-1 convolutions whose input
 * channel count is a multiple of 64 run on the kernel that keeps a tile's input and halo in LDS; 0 sends them to the
 * implicit-GEMM kernel like every other convolution.  Returns the previous value; any other argument only queries. */
int pd_set_conv_halo(int32_t on);

/* How many executed ops a stage remembers for pd_stage_trace: the most recent `max_ops` (default 65536; 0 switches
 * the record off and clears it).  Host-side only. */
int pd_stage_set_trace_limit(pd_stage* st, size_t max_ops);

/* The recurrence of an LSTM layer.  multi_step != 0 (the default): layers whose grid of 16 x 16 tiles (rows x hidden
 * units) fits the chip, with hidden size <= 1024, run all time steps of a pass in ONE launch whose workgroups exchange
 * the hidden state (forward) or the gate gradients (backward) through memory and wait for each other's results per step
 * with BOUNDED polling; other layers, and everything under stream capture, take one launch per time step.
 * multi_step = 0: one launch per time step always.  Results are bit-identical either way.
 * Measured on MI355X (hidden 1000, minibatch 64, 80 steps): 5.6 against 7.8 us per step for a stage on its own (1.29
 * against 1.65 ms per F + B + U); 4.15 ms per minibatch either way for the two-stage pipeline on one GPU, where such a
 * launch keeps the other stage's kernels off the chip for its duration and per-step launches of two stages interleave.
 * spin_limit: fetches before a wave gives up waiting for its peers' results (0: the default of 4,000,000); starve != 0:
 * no workgroup publishes its results, so that no wait can succeed -- for testing that the launch still ends and that
 * the failure is reported (PD_ESTATE from pd_stage_check or the stage's next synchronising call).  Returns the old
 * multi_step setting.  Process-wide, not thread-safe. */
int pd_set_recurrence_kernel(int32_t multi_step, uint32_t spin_limit, uint32_t starve);

#ifdef __cplusplus
}
#endif
#endif /* PD_DEBUG_H_ */
