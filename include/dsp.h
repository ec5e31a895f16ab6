/*
 * dsp.h -- C ABI of the MI355X (gfx950) library for the per-block training step of
 * Diversely Stale Parameters (DSP).
 *
 * Vocabulary follows the paper.  A CNN is split into K consecutive blocks
 * h_{k+1} = f_k(h_k; x_k) with loss L(h_K, l) (Section 2, Eq. (1)).  In the batch pipeline
 * DSP(p_0..p_{K-1}; m_0..m_{K-1}) (Section 3.3, Appendix A) block k, at every tick,
 *   1. runs the forward pass of the newest mini-batch a on its current parameters and stores
 *      the block INPUT h_k(a) (queue M_k, 1+m_k entries; no activations, no weight copies),
 *   2. recomputes f_k on the input h_k(b) it stored m_k mini-batches earlier, with the SAME
 *      current parameters, and back-propagates the delayed error gradient G_{h_{k+1}}(b)
 *      (Section 3.2, Eq. (5)): G_{x_k}(b), G_{h_k}(b),
 *   3. applies a momentum-SGD update (Section 2, Eq. (3) with s = 0).
 * m_k is the layer-wise staleness of block k (Section 3.1): m_k updates separate the forward
 * and the backward use of x_k for one mini-batch.
 *
 * Conventions
 *   - Every function returns a dsp_status; nothing throws or aborts across this boundary.
 *   - "d_" pointers are DEVICE pointers on the current HIP device, "h_" pointers are HOST
 *     pointers.  Streams are hipStream_t passed as void* (NULL = the null stream).
 *   - Activations and error gradients cross the boundary in NHWC order in the block's
 *     storage type (float for DSP_FP32, bfloat16 for DSP_BF16); tensors after a global
 *     average pool (N x C) and the loss are always float.
 *   - Parameters cross the boundary on the HOST as float in "layer order": for each layer in
 *     turn, conv: w[cout][cin][r][s]; bn: gamma[c], beta[c]; linear: W[cout][cin], c[cout].
 *   - The library allocates device memory only in the *_init calls and in
 *     dsp_pipeline_attach_gradient_probe / dsp_pipeline_set_forward_streams (first step after it);
 *     the step calls launch kernels asynchronously on the given stream and allocate nothing.
 *   - Arguments are checked before anything is launched: DSP_EINVAL and DSP_ESTATE leave the
 *     object as it was.  DSP_EHIP or DSP_ENOMEM out of a step call may have launched part of the
 *     step: the object's contents are then unspecified and it should be destroyed.
 *   - Objects are not thread-safe; calls on one block must be issued in pipeline order
 *     (forward, then recompute_backward, then param_update) or DSP_ESTATE is returned.
 */
#ifndef DSP_H
#define DSP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum dsp_status {
    DSP_OK = 0,
    DSP_EINVAL = 1, /* bad argument / descriptor / schedule (Appendix A violated) */
    DSP_ESTATE = 2, /* call out of pipeline order */
    DSP_ENOMEM = 3, /* device or host allocation failed */
    DSP_EHIP = 4    /* a HIP runtime call failed; see dsp_last_error() */
} dsp_status;

typedef enum dsp_dtype {
    DSP_FP32 = 0, /* fp32 storage, fp32 MFMA */
    DSP_BF16 = 1  /* bf16 storage of activations/gradients/shadow weights, bf16 MFMA with fp32
                     accumulation; fp32 master weights, momentum, weight gradients, BN statistics */
} dsp_dtype;

typedef enum dsp_op {
    DSP_OP_CONV = 0,      /* cross-correlation, zero padding, no bias */
    DSP_OP_BN = 1,        /* training-mode batch norm [+ residual add] [+ ReLU] */
    DSP_OP_MAXPOOL = 2,   /* r x r window, stride, pad (-inf padding, first maximum wins) */
    DSP_OP_GAP = 3,       /* global average pool over H, W */
    DSP_OP_LINEAR = 4,    /* z = W h + c */
    DSP_OP_SOFTMAX_CE = 5, /* L = mean over the batch of -log softmax(z)[label]; last block only */
    DSP_OP_ADD = 6         /* y = in0 + in1, two feature maps of one shape (shortcut of a pre-activation unit) */
} dsp_op;

/* One layer of a block.  Layer i produces tensor i; in0 = -1 names the block input h_k. */
typedef struct dsp_layer_desc {
    int32_t op;     /* dsp_op */
    int32_t in0;    /* producer of the input: layer index, or -1 for the block input */
    int32_t in1;    /* BN: tensor added after normalisation (residual), or -2 for none; ADD: the second operand */
    int32_t cin;    /* conv/linear input channels; BN channels */
    int32_t cout;   /* conv/linear output channels */
    int32_t r, s;   /* conv filter height/width; maxpool window (r) */
    int32_t stride; /* conv/maxpool stride */
    int32_t pad;    /* conv/maxpool padding */
    int32_t relu;   /* BN only: apply ReLU after (BN + residual) */
    int32_t groups; /* conv only: > 1 makes it a grouped convolution (aggregated transforms of ResNeXt): group g maps
                       input channels [g cin/groups, (g+1) cin/groups) to output channels [g cout/groups, ...) with
                       filters [cout][r][s][cin/groups]; 0 and 1 both mean an ordinary convolution */
} dsp_layer_desc;

/* One block of the split CNN and its place in DSP(p; m). */
typedef struct dsp_block_desc {
    int32_t n_layers;
    const dsp_layer_desc* layers;
    int32_t N, C, H, W;       /* mini-batch size and shape of the block input h_k */
    int32_t dtype;            /* dsp_dtype */
    int32_t k, K;             /* index of this block, number of blocks */
    int32_t m_k;              /* layer-wise staleness: the stored-input queue M_k has 1+m_k entries */
    int32_t p_prev;           /* p_{k-1} (0 for a stand-alone block): the output queue P_{k-1} of the block
                                 below is fused into M_k, which then has 1+m_k+p_prev entries, so the
                                 producer writes h_k straight into its slot (no copy between queues).
                                 p_prev = p_{k-1} + spare gives the queue `spare` entries of slack
                                 (see dsp_pipeline_init); results do not depend on it */
    int32_t needs_input_grad; /* 0 for the block that reads the data h_0 (q_0 = 0): G_{h_0} is not formed */
    float bn_eps;
} dsp_block_desc;

typedef struct dsp_block dsp_block;
typedef struct dsp_pipeline dsp_pipeline;

/* ---- schedule (host only; Section 3.3 and Appendix A) ------------------------------------ */

/*
 * Validates DSP(p; m) and writes q_k = m_{k-1} - p_{k-1} - m_k (q_0 = 0) into q[K].
 * Accepted: p_k > 0 for k < K-1, p_{K-1} = 0, m_k > 0 for k < K-1, m_{K-1} >= 0 (the paper's own
 * schedules end in m = 0), q_k > 0 for k >= 1; or the all-zero schedule, which is ordinary
 * backpropagation (Section 3.1, remark a; with K blocks: the model-parallel BP of Section 6); or every
 * p_k = 0 with m_k > 0 for k < K-1 and q_k > 0: forward-locked, stale backward passes -- with
 * m_k = K-1-k the schedule of the features-replay comparison of Section 6 (the pipeline then orders the
 * forward passes of a tick block after block).  Anything else: DSP_EINVAL.
 */
int dsp_schedule_validate(int32_t K, const int32_t* p, const int32_t* m, int32_t* q);

/*
 * Closed-form position of block k at tick tau: forward mini-batch a = tau - sum_{j<k} p_j,
 * backward mini-batch b = a - m_k (either is -1 while the pipeline fills), the number of updates
 * already applied to x_k (= max(0, b)), and the queue slots: M_k slot of a and of b (ring of
 * 1+m_k+p_{k-1} entries), Q_k slot written for b (ring of 1+q_k entries; -1 for k = 0) and the
 * Q_{k+1} slot read for b (-1 for the last block).  out[7] = {a, b, version, slot_fwd, slot_bwd,
 * q_write_slot, q_read_slot}.
 */
int dsp_schedule_index(int32_t K, const int32_t* p, const int32_t* m, int32_t k, int64_t tau, int64_t out[7]);

/* Queue memory in ELEMENTS for per-block boundary sizes h_elems[k] = |h_k|, k = 0..K (Section 3.3:
 * space O(L + sum_k (m_k + p_k + q_k))): sum_k (1+m_k+p_{k-1}) |h_k| + (1+q_k) |h_k| [k >= 1]. */
int dsp_schedule_queue_elems(int32_t K, const int32_t* p, const int32_t* m, const int64_t* h_elems,
                             int64_t* total);

/*
 * Cross-block ordering of DSP(p; m) when the queues between blocks k-1 and k hold spare[k] entries
 * beyond the minimum (spare may be NULL = all 0; spare[0] must be 0; each 0..64): block k may start
 * tick tau once block k-1 has finished tick tau - wait_down[k] and block k+1 tick tau - wait_up[k]
 * (0 = no such neighbour, or an all-zero schedule), where wait_down[k] = min(p_{k-1}, 1 + spare[k])
 * and wait_up[k] = min(q_{k+1}, 1 + spare[k+1]): the nearer of the tick that wrote what the block
 * reads and the tick that last read what it overwrites.  *label_slots (may be NULL) = mini-batches
 * of labels a data source feeding block 0 must keep for the last block.  Host only.
 */
int dsp_schedule_waits(int32_t K, const int32_t* p, const int32_t* m, const int32_t* spare, int32_t* wait_down,
                       int32_t* wait_up, int32_t* label_slots);

/* ---- one block (Section 2 Eq. (1)-(3), Section 3.2 Eq. (5)) ------------------------------ */

/*
 * Builds block k: checks the layer graph, copies h_params (n_params floats, layer order) to the
 * device, zeroes the momentum, sets the update counter ("parameter version") to 0 and allocates
 * the stored-input ring, the recompute workspace and the gradient buffers.  *out owns them.
 */
int dsp_block_init(const dsp_block_desc* desc, const float* h_params, size_t n_params, dsp_block** out);
int dsp_block_destroy(dsp_block* b);

/*
 * Forward pass of mini-batch batch_id on the current parameters (Eq. (5), third line: what
 * flows upward is produced by forward parameters).  batch_id must be the next id in order
 * (0, 1, 2, ...).  Stores the input into ring slot batch_id mod ring_entries (no copy if d_in
 * already is dsp_block_input_slot(batch_id)), writes h_{k+1}(batch_id) to d_out (may be NULL
 * for the last block).  Last block with a softmax_ce layer: d_labels = int32[N] labels,
 * d_loss = one float receiving the mini-batch loss; its own G_{h_K} is kept for the backward.
 */
int dsp_block_forward(dsp_block* b, int64_t batch_id, const void* d_in, void* d_out, const int32_t* d_labels,
                      float* d_loss, void* stream);

/*
 * Eq. (5), lines 1-2: recomputes f_k on the stored input h_k(batch_id) with the CURRENT parameters
 * and back-propagates d_grad_out = G_{h_{k+1}}(batch_id) (NULL: the block's own loss gradient).
 * batch_id must equal (latest forward id) - m_k and follow the previous backward id.  Writes
 * G_{h_k} to d_grad_in (ignored when needs_input_grad = 0) and leaves G_{x_k} in a library buffer
 * for dsp_param_update.  With m_k = 0 the forward pass just run is reused instead of recomputed.
 */
int dsp_block_recompute_backward(dsp_block* b, int64_t batch_id, const void* d_grad_out, void* d_grad_in,
                                 void* stream);

/*
 * dsp_block_forward(batch_fwd, ...) followed by dsp_block_recompute_backward(batch_bwd, ...) as one
 * call, with the same arguments, checks and results (bit-identical).  Both forward sweeps of a tick --
 * the current mini-batch and the recompute of the stale one -- evaluate f_k with the same parameters
 * (Section 3: the update comes after both), so for m_k > 0 every layer serves both with one kernel
 * launch that carries two problem instances; this needs the second buffer set of
 * dsp_block_enable_forward_lane, which the first call allocates.  batch_bwd must be
 * batch_fwd - m_k >= 0; dsp_param_update still follows.
 */
int dsp_block_step(dsp_block* b, int64_t batch_fwd, const void* d_in, void* d_out, const int32_t* d_labels, float* d_loss,
                   int64_t batch_bwd, const void* d_grad_out, void* d_grad_in, void* stream);

/*
 * Stochastic unified momentum, Eq. (3), for s = 0 (heavy ball) and s = 1 (Nesterov), in velocity
 * form: with G' = G + weight_decay * x (conv/linear weights only),
 *     v <- momentum * v + G',   x <- x - lr * v                      (s = 0)
 *     v <- momentum * v + G',   x <- x - lr * (G' + momentum * v)    (s = 1)
 * which is the (y, y^s) recursion of Eq. (3) with y^{s,0} = x^0, v^0 = 0 and v^n = -(x^n - x^{n-1}) / lr
 * for s = 0, v^n = -(y^n - y^{n-1}) / lr for s = 1.
 * The block remembers the step size of its previous update; when lr differs from it, v is first
 * multiplied by (previous lr / lr), so that the momentum term stays the difference of iterates that
 * Eq. (3) prescribes under a learning-rate schedule.  lr = 0 leaves x unchanged, which is what Eq. (3)
 * gives as long as no momentum is carried (momentum = 0, or no update with lr > 0 so far: the probe
 * pipeline of dsp_pipeline_attach_gradient_probe); a step of size 0 AFTER updates with lr > 0 and
 * momentum != 0 would still have to move x by momentum * (x^n - x^{n-1}), which the velocity form cannot
 * express, and is refused (DSP_EINVAL, nothing consumed).  Other values of s need the previous gradient
 * and are refused (DSP_EINVAL).
 * Consumes the pending G_{x_k} exactly once (DSP_ESTATE if there is none) and increments the
 * update counter.  dsp_param_update is the s = 0 case.
 */
int dsp_param_update_sum(dsp_block* b, float lr, float momentum, int32_t s, float weight_decay, void* stream);
int dsp_param_update(dsp_block* b, float lr, float momentum, float weight_decay, void* stream);

/*
 * Allocates a second set of the buffers a forward pass writes.  Afterwards dsp_block_forward no
 * longer touches anything dsp_block_recompute_backward reads or writes, so the two calls of one
 * tick may be enqueued on different streams: the forward of mini-batch a and the backward of
 * mini-batch a - m_k use the same parameters and are independent until the update (Section 3,
 * Figure 2).  The caller must order both before dsp_param_update, and the next dsp_block_forward
 * after that update.  Results are bit-identical to the single-stream order.  Only for m_k > 0
 * (DSP_EINVAL otherwise: with m_k = 0 the backward reuses the forward's activations); calling it
 * again is a no-op.  The extra memory shows up in dsp_block_memory's workspace figure.
 */
int dsp_block_enable_forward_lane(dsp_block* b);

/* Device address of the M_k ring slot that will hold h_k(batch_id). */
int dsp_block_input_slot(dsp_block* b, int64_t batch_id, void** d_slot);

/* out[8] = {updates applied, next forward id, next backward id, ring entries, pending gradient (0/1),
 * parameter count, update count at the forward of the batch whose backward comes next (-1 if none),
 * slot of that batch}. */
int dsp_block_query(const dsp_block* b, int64_t out[8]);
/* Shape (N, C, H, W) of h_{k+1}; H = W = 1 after a pool/linear layer.  out[4] = 1 if it is float
 * whatever the block dtype (behind a global average pool), else 0. */
int dsp_block_output_shape(const dsp_block* b, int32_t out[5]);
/* Shape (N, C, H, W) of h_k and the block dtype: out[5] = {N, C, H, W, dtype}. */
int dsp_block_input_shape(const dsp_block* b, int32_t out[5]);
/* Bytes held on the device: stored-input ring, workspace (activations + gradients), parameters. */
int dsp_block_memory(const dsp_block* b, size_t* ring_bytes, size_t* workspace_bytes, size_t* param_bytes);

/* Host <-> device state in layer order (synchronous; they synchronise the device first). */
int dsp_block_get_params(dsp_block* b, float* h_dst, size_t n);
int dsp_block_set_params(dsp_block* b, const float* h_src, size_t n);
int dsp_block_get_momentum(dsp_block* b, float* h_dst, size_t n);
int dsp_block_set_momentum(dsp_block* b, const float* h_src, size_t n);
int dsp_block_get_grads(dsp_block* b, float* h_dst, size_t n);

/* ---- K blocks on K HIP streams of one GPU (Section 3.3) ---------------------------------- */

/*
 * Wires K blocks (built with matching k, K, m_k, p_prev = p_{k-1}) into DSP(p; m): one stream per
 * block, gradient rings Q_k of 1+q_k entries, a label ring, a loss history of max_ticks floats.
 * The blocks stay owned by the caller and must outlive the pipeline.
 * Spare queue entries: a block k >= 1 built with p_prev = p_{k-1} + spare_k (0 <= spare_k <= 64) has
 * spare_k more ring entries than the schedule needs; Q_k then gets spare_k more as well, and the two
 * blocks k-1 and k may drift apart by more than one tick (block k-1 waits for tick
 * tau - min(q_k, 1+spare_k) of block k, block k for tick tau - min(p_{k-1}, 1+spare_k) of block k-1)
 * instead of running in lockstep: the slack that the FIFO queues of Section 6 ("Robustness") give a
 * block whose neighbour is late.  Which mini-batch meets which parameters depends on the tick number
 * only, so every result is bit-identical with and without spare entries.  A smaller ring, or a larger
 * one in block 0: DSP_EINVAL.
 */
int dsp_pipeline_init(int32_t K, dsp_block* const* blocks, const int32_t* p, const int32_t* m, float lr,
                      float momentum, float weight_decay, int64_t max_ticks, dsp_pipeline** out);
int dsp_pipeline_destroy(dsp_pipeline* pl);

/*
 * One tick: feeds mini-batch number tau (d_batch: NHWC block-0 input, d_labels: int32[N], both
 * ready on `stream`); every block k with a >= 0 runs forward(a), then, if b >= 0,
 * recompute_backward(b) and its update, on its own stream.  Blocks never depend on each other
 * inside a tick; across ticks each stream waits for its neighbours' previous tick (an earlier one
 * where the queues have spare entries, see dsp_pipeline_init).  On return
 * `stream` is ordered after the copies of d_batch/d_labels, so the caller may refill them.
 * If h_loss != NULL the call blocks until the loss of this tick is known and returns it with
 * its mini-batch id (*loss_batch_id = -1 while the pipeline fills); pass NULL to stay asynchronous
 * and read the history later with dsp_pipeline_losses().
 */
int dsp_pipeline_step(dsp_pipeline* pl, const void* d_batch, const int32_t* d_labels, float* h_loss,
                      int64_t* loss_batch_id, void* stream);

/*
 * Step size, momentum constant, s of Eq. (3) (0 or 1) and weight decay used by the updates of all
 * later ticks (a step learning-rate schedule calls this between steps; dsp_pipeline_init sets s = 0).
 */
int dsp_pipeline_set_optimizer(dsp_pipeline* pl, float lr, float momentum, int32_t s, float weight_decay);

/*
 * Gradient-difference diagnostic (Lemma 1; the quantity plotted in Section 5.4).  `probe` is a second
 * pipeline over K blocks of the same architecture, built with the all-zero schedule (ordinary
 * backpropagation), step size 0 and max_ticks >= pl's; it stays owned by the caller and must outlive
 * pl's last step.  Call once, before the first step of either pipeline.  From then on every
 * dsp_pipeline_step(pl) (labels required) additionally
 *   - keeps, per block, the parameters it runs the forward pass of mini-batch a = tau - P_k with,
 *   - keeps the DSP gradient G_{x_k} of mini-batch b_k = a - m_k,
 *   - and, once block 0 has formed its gradient of mini-batch b (the last block to do so), loads the
 *     kept forward-time parameters of b into the probe blocks, back-propagates h_0(b) through them and
 *     forms, per block, sum (G^DSP_{x_k} - G^BP_{x_k})^2 and sum (G^BP_{x_k})^2 in fp64.
 * The step then synchronises all streams several times and never replays graphs: a diagnostic mode,
 * not a timed path.  Costs device memory for (1 + m_0 - P_k) parameter copies and
 * (1 + m_0 - P_k - m_k) gradient copies per block.
 */
int dsp_pipeline_attach_gradient_probe(dsp_pipeline* pl, dsp_pipeline* probe);
/*
 * Result of the latest step: *batch_id = the mini-batch evaluated (-1: none yet, while block 0 has no
 * gradient), diff_sumsq[K] and bp_sumsq[K] (host) as defined above.
 */
int dsp_pipeline_gradient_difference(dsp_pipeline* pl, int64_t* batch_id, double* diff_sumsq, double* bp_sumsq);

/*
 * How the launches of a tick reach the GPU (results are bit-identical in every mode):
 *  - launch threads (default on): the chain of block k >= 1 is issued by a host thread of its own while
 *    the caller's thread issues block 0; the call returns when every chain has been enqueued.
 *  - graph replay (default off): steady-state ticks are recorded once per ring position into HIP graphs
 *    and replayed with one launch each.
 */
int dsp_pipeline_set_launch_threads(dsp_pipeline* pl, int32_t enable);
/*
 *  - single stream (default off): the K chains of a tick are issued one after the other on ONE stream by the
 *    caller's thread, so no two kernels overlap: the mode in which a per-kernel duration is that kernel's own
 *    (measurement support; blocks within a tick are independent, so any issue order gives the same bits).
 *    Synchronises the pipeline's streams when called; may be changed between steps; not with forward streams.
 */
int dsp_pipeline_set_single_stream(dsp_pipeline* pl, int32_t enable);
int dsp_pipeline_set_graph_replay(dsp_pipeline* pl, int32_t enable);
/*
 *  - forward streams (default off): a block with m_k > 0 runs the forward pass of the current
 *    mini-batch on a second stream, concurrently with the recompute + backward of the stale one
 *    (dsp_block_enable_forward_lane); the update waits for both.  Must be set before the first
 *    dsp_pipeline_step (DSP_ESTATE afterwards); not available with spare queue entries (DSP_EINVAL).
 */
int dsp_pipeline_set_forward_streams(dsp_pipeline* pl, int32_t enable);
/*
 *  - twin launches (default on): once a block runs both a forward and a backward in a tick it uses
 *    dsp_block_step, i.e. one launch per layer for the forward of the current mini-batch and the
 *    recompute of the stale one.  Ignored for blocks that use a forward stream.  May be changed
 *    between steps.
 */
int dsp_pipeline_set_twin_launches(dsp_pipeline* pl, int32_t enable);
/* Straggler emulation: block k's stream spins for `microseconds` before its work in every later tick
 * (0 <= microseconds <= 1000000; may be changed between steps at no cost unless graph replay is on). */
int dsp_pipeline_set_delay(dsp_pipeline* pl, int32_t k, int32_t microseconds);
/* Waits for all K streams. */
int dsp_pipeline_sync(dsp_pipeline* pl);
/* Copies the losses of mini-batches [0, n) to h_dst after a sync; n <= number of losses produced. */
int dsp_pipeline_losses(dsp_pipeline* pl, float* h_dst, int64_t n, int64_t* n_available);
/* Number of ticks issued so far. */
int dsp_pipeline_ticks(const dsp_pipeline* pl, int64_t* ticks);

/* ---- single-layer entry points (used by the kernel parity tests and micro-benchmarks) ------ */

/*
 * Convolution kernels on NHWC device tensors of type `dtype`; filters in the library's layout:
 * d_w  = w[cout][r][s][cin] (forward / backward-weight), d_wt = w[cin][R-1-r][S-1-s][cout]
 * (backward-data, stride 1).  Backward-data of a stride-2 layer runs as four dense problems, one per parity
 * class (hi % 2, wi % 2) of the input pixel, and takes d_wt class by class: classes in the order (0,0), (0,1),
 * (1,0), (1,1); class (ph, pw) holds [cin][j][l][cout] for the taps r' = r0 + 2 j, s' = s0 + 2 l of the flipped
 * filter w[cin][r'][s'][cout], r0 = (R-1-pad - ph) mod 2, s0 = (S-1-pad - pw) mod 2 (the same elements, reordered).  dsp_conv_workspace_bytes() sizes d_workspace for backward-weight (split
 * reduction partials).  accumulate != 0 adds into d_dx instead of overwriting.
 */
int dsp_conv_forward(int32_t dtype, const void* d_x, const void* d_w, void* d_y, int32_t N, int32_t H, int32_t W,
                     int32_t cin, int32_t cout, int32_t r, int32_t s, int32_t stride, int32_t pad, void* stream);
int dsp_conv_backward_data(int32_t dtype, const void* d_dy, const void* d_wt, void* d_dx, int32_t N, int32_t H,
                           int32_t W, int32_t cin, int32_t cout, int32_t r, int32_t s, int32_t stride, int32_t pad,
                           int32_t accumulate, void* stream);
int dsp_conv_backward_weight(int32_t dtype, const void* d_x, const void* d_dy, float* d_dw, int32_t N, int32_t H,
                             int32_t W, int32_t cin, int32_t cout, int32_t r, int32_t s, int32_t stride,
                             int32_t pad, void* d_workspace, size_t workspace_bytes, void* stream);
int dsp_conv_workspace_bytes(int32_t N, int32_t H, int32_t W, int32_t cin, int32_t cout, int32_t r, int32_t s,
                             int32_t stride, int32_t pad, size_t* bytes);

/*
 * The same three kernels for a grouped convolution (the aggregated transforms of ResNeXt-29, one of the networks of
 * the paper's speed-up table): `groups` divides cin and cout; group g maps input channels [g cin/groups,
 * (g+1) cin/groups) to output channels [g cout/groups, (g+1) cout/groups).  Tensors keep all cin (cout) channels per
 * pixel.  d_w = w[cout][r][s][cin/groups] (the output channel selects the group); d_wt (stride 1) =
 * w[g cin/groups + ci][R-1-r][S-1-s][co within the group]: cin rows of r*s*cout/groups elements; for stride 2 the
 * same class-by-class order as above with these rows and runs.  d_dw has the layout of d_w.  groups = 1 is the
 * ordinary convolution.  Errors: DSP_EINVAL if groups does not divide the channel counts, else as above.
 */
int dsp_grouped_conv_forward(int32_t dtype, const void* d_x, const void* d_w, void* d_y, int32_t N, int32_t H, int32_t W,
                             int32_t cin, int32_t cout, int32_t r, int32_t s, int32_t stride, int32_t pad, int32_t groups,
                             void* stream);
int dsp_grouped_conv_backward_data(int32_t dtype, const void* d_dy, const void* d_wt, void* d_dx, int32_t N, int32_t H,
                                   int32_t W, int32_t cin, int32_t cout, int32_t r, int32_t s, int32_t stride, int32_t pad,
                                   int32_t groups, int32_t accumulate, void* stream);
int dsp_grouped_conv_backward_weight(int32_t dtype, const void* d_x, const void* d_dy, float* d_dw, int32_t N, int32_t H,
                                     int32_t W, int32_t cin, int32_t cout, int32_t r, int32_t s, int32_t stride, int32_t pad,
                                     int32_t groups, void* d_workspace, size_t workspace_bytes, void* stream);
int dsp_grouped_conv_workspace_bytes(int32_t N, int32_t H, int32_t W, int32_t cin, int32_t cout, int32_t r, int32_t s,
                                     int32_t stride, int32_t pad, int32_t groups, size_t* bytes);

/*
 * The other layers of a block (the paper names networks, not layers; these are the textbook definitions
 * the block function f_k of Eq. (1) and its chain rule, Eq. (2), are assembled from), each as the kernels
 * the block engine launches for it, on caller-owned device tensors.  Feature maps are NHWC in `dtype`
 * seen as x[M][C], M = N*H*W rows; everything behind a global average pool is float.
 *
 * Batch norm in training mode over the M rows, per channel: mean, biased variance, y = [relu](gamma *
 * (x - mean) / sqrt(var + eps) + beta [+ res]); d_mean / d_invstd (C floats each) receive the statistics
 * the backward needs.  Backward: dz = dy * [y > 0] (relu) ; dres (+)= dz; dgamma = sum dz * xhat;
 * dbeta = sum dz; dx (+)= gamma * invstd * (dz - dbeta / M - xhat * dgamma / M).  d_res / d_dres may be NULL.
 * d_workspace: dsp_bn_workspace_bytes(C) bytes, 16-byte aligned, contents unspecified before and after.
 */
int dsp_bn_workspace_bytes(int32_t C, size_t* bytes);
int dsp_bn_forward(int32_t dtype, const void* d_x, const void* d_res, void* d_y, const float* d_gamma, const float* d_beta,
                   float eps, int64_t M, int32_t C, int32_t relu, float* d_mean, float* d_invstd, void* d_workspace,
                   size_t workspace_bytes, void* stream);
int dsp_bn_backward(int32_t dtype, const void* d_dy, const void* d_x, const void* d_y, void* d_dx, void* d_dres,
                    int32_t dres_accumulate, int32_t dx_accumulate, const float* d_gamma, const float* d_mean,
                    const float* d_invstd, float* d_dgamma, float* d_dbeta, int64_t M, int32_t C, int32_t relu,
                    void* d_workspace, size_t workspace_bytes, void* stream);
/*
 * The two forms a block uses where a batch norm + ReLU has no residual (same definitions as above, fewer passes over
 * memory; device pointers throughout, errors as above):
 * dsp_bn_relu_maxpool_forward -- batch norm + ReLU whose only reader is a max pool (k x k window, k <= 4, -inf padding,
 *   first maximum wins; bf16 tensors with C % 8 == 0 only, else DSP_EINVAL): d_pool[N][Ho][Wo][C] and d_argmax (one byte
 *   per output element, r * k + s) are the bits dsp_bn_forward(relu = 1) followed by dsp_maxpool_forward leave; the
 *   normalised tensor itself is never written.  d_scale_shift (2 * C floats, 16-byte aligned) receives the per-channel
 *   {scale[C], shift[C]} the output was formed with: y = relu(round(fma(x, scale, shift))).
 * dsp_bn_relu_backward_from_x -- dsp_bn_backward(relu = 1, no residual) without reading y: the ReLU decision [y > 0] is
 *   taken by forming y from x and the forward pass's d_scale_shift again, with the forward kernel's own expression and
 *   rounding, so dx, dgamma and dbeta are the bits dsp_bn_backward leaves when given the stored y.
 * dsp_bn_relu_maxpool_backward -- the backward of dsp_bn_relu_maxpool_forward in two passes over x: the gradient the
 *   pool hands to each pixel (the sum of d_dpool over the windows whose recorded tap in d_argmax is that pixel, rounded
 *   to the storage type, as dsp_maxpool_backward stores it) is formed inside the batch-norm kernels instead of being
 *   stored.  Every masked gradient is the one dsp_maxpool_backward + dsp_bn_backward work on; the per-channel sums are
 *   taken in another order, so dgamma, dbeta and dx agree with that pair to double-rounding noise (relative 1e-6), not
 *   bit for bit.  bf16, C % 8 == 0, k = 3, stride = 2, pad = 1, even H and W only, else DSP_EINVAL.
 */
/*
 * Batch norm + ReLU WITH a residual input, as a block runs it: dsp_bn_forward_bits is dsp_bn_forward(relu = 1) that also
 * leaves, in d_relu_bits (dsp_bn_relu_bits_bytes() bytes: one per channel vector of 16 bytes; channel counts that are no
 * whole number of vectors are refused with DSP_EINVAL), bit k of byte v = element k of vector v of y as stored is positive;
 * dsp_bn_backward_bits is dsp_bn_backward(relu = 1) that takes its ReLU decisions from those bytes instead of reading y:
 * the same bits in dx, dres, dgamma, dbeta, one tensor pass less in each of its two kernels.
 */
int dsp_bn_relu_bits_bytes(int32_t dtype, int64_t M, int32_t C, size_t* bytes);
int dsp_bn_forward_bits(int32_t dtype, const void* d_x, const void* d_res, void* d_y, const float* d_gamma, const float* d_beta,
                        float eps, int64_t M, int32_t C, float* d_mean, float* d_invstd, uint8_t* d_relu_bits, void* d_workspace,
                        size_t workspace_bytes, void* stream);
int dsp_bn_backward_bits(int32_t dtype, const void* d_dy, const void* d_x, const uint8_t* d_relu_bits, void* d_dx, void* d_dres,
                         int32_t dres_accumulate, int32_t dx_accumulate, const float* d_gamma, const float* d_mean,
                         const float* d_invstd, float* d_dgamma, float* d_dbeta, int64_t M, int32_t C, void* d_workspace,
                         size_t workspace_bytes, void* stream);
int dsp_bn_relu_maxpool_forward(int32_t dtype, const void* d_x, const float* d_gamma, const float* d_beta, float eps, int32_t N,
                                int32_t H, int32_t W, int32_t C, int32_t k, int32_t stride, int32_t pad, void* d_pool,
                                uint8_t* d_argmax, float* d_mean, float* d_invstd, float* d_scale_shift, void* d_workspace,
                                size_t workspace_bytes, void* stream);
int dsp_bn_relu_backward_from_x(int32_t dtype, const void* d_dy, const void* d_x, const float* d_scale_shift, void* d_dx,
                                int32_t dx_accumulate, const float* d_gamma, const float* d_mean, const float* d_invstd,
                                float* d_dgamma, float* d_dbeta, int64_t M, int32_t C, void* d_workspace, size_t workspace_bytes,
                                void* stream);
int dsp_bn_relu_maxpool_backward(int32_t dtype, const void* d_dpool, const uint8_t* d_argmax, const void* d_x,
                                 const float* d_scale_shift, void* d_dx, int32_t dx_accumulate, const float* d_gamma,
                                 const float* d_mean, const float* d_invstd, float* d_dgamma, float* d_dbeta, int32_t N, int32_t H,
                                 int32_t W, int32_t C, int32_t k, int32_t stride, int32_t pad, void* d_workspace,
                                 size_t workspace_bytes, void* stream);
/* k x k max pool (padding = -inf, the first maximum in row-major window order wins); d_argmax keeps one
 * byte per output element (window position r*k+s); backward: dx (+)= the dy of every window that chose the pixel. */
int dsp_maxpool_forward(int32_t dtype, const void* d_x, void* d_y, uint8_t* d_argmax, int32_t N, int32_t H, int32_t W,
                        int32_t C, int32_t k, int32_t stride, int32_t pad, void* stream);
int dsp_maxpool_backward(int32_t dtype, const void* d_dy, const uint8_t* d_argmax, void* d_dx, int32_t accumulate, int32_t N,
                         int32_t H, int32_t W, int32_t C, int32_t k, int32_t stride, int32_t pad, void* stream);
/* y = a + b over n elements; backward: da (+)= dy and, unless d_db is NULL, db (+)= dy. */
int dsp_add_forward(int32_t dtype, const void* d_a, const void* d_b, void* d_y, int64_t n, void* stream);
int dsp_add_backward(int32_t dtype, const void* d_dy, void* d_da, int32_t da_accumulate, void* d_db, int32_t db_accumulate,
                     int64_t n, void* stream);
/* y[n][c] = mean over the HW positions of x[n][.][c] (float); backward: dx (+)= dy / HW. */
int dsp_gap_forward(int32_t dtype, const void* d_x, float* d_y, int32_t N, int32_t HW, int32_t C, void* stream);
int dsp_gap_backward(int32_t dtype, const float* d_dy, void* d_dx, int32_t accumulate, int32_t N, int32_t HW, int32_t C,
                     void* stream);
/* z = x W^T + bias with W[cout][cin]; backward: dx = dz W (skipped if d_dx is NULL), dW = dz^T x, dbias = sum_n dz. */
int dsp_linear_forward(const float* d_x, const float* d_w, const float* d_bias, float* d_z, int32_t N, int32_t cin,
                       int32_t cout, void* stream);
int dsp_linear_backward(const float* d_x, const float* d_w, const float* d_dz, float* d_dx, float* d_dw, float* d_dbias,
                        int32_t N, int32_t cin, int32_t cout, void* stream);
/* L(h_K, l) of Eq. (1): *d_loss = mean_n -log softmax(z_n)[label_n], d_dz = dL/dz; d_row_loss: N floats of scratch. */
int dsp_softmax_ce(const float* d_z, const int32_t* d_labels, float* d_loss, float* d_dz, float* d_row_loss, int32_t N,
                   int32_t C, void* stream);

/*
 * Test support: copies what layer `layer` of the block left in the buffers the backward sweep reads (the
 * recompute of the latest dsp_block_recompute_backward / dsp_block_step, or the latest forward when m_k = 0)
 * to the host after a device synchronisation: the layer's output in the block's storage type (NHWC; float
 * behind a pool), `bytes` = its exact size; for a max-pool layer dsp_block_get_pool_argmax copies the chosen
 * window positions (one byte per output element).  These are the values the ReLU masks and pooling
 * decisions of the backward sweep were taken on.
 */
int dsp_block_get_activation(dsp_block* b, int32_t layer, void* h_dst, size_t bytes);
int dsp_block_get_pool_argmax(dsp_block* b, int32_t layer, uint8_t* h_dst, size_t bytes);

/*
 * dsp_conv_backward_weight for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * kernels and bits as dsp_conv_backward_weight, but the split-reduction partials live in a fixed buffer
 * inside the loaded library (dsp_conv_backward_weight_static_bytes() bytes, 16 MiB, held on every GPU the
 * library runs on until the process ends); the call allocates nothing.  A layer whose partials
 * (dsp_conv_workspace_bytes) exceed that size is refused with DSP_EINVAL before anything is launched.
 * All calls on one GPU share the buffer: calls that overlap in time on one GPU (two streams, two threads)
 * race and must be ordered by the caller.  Nothing in the buffer has to start at zero, so it is never cleared.
 */
int dsp_conv_backward_weight_static(int32_t dtype, const void* d_x, const void* d_dy, float* d_dw, int32_t N, int32_t H,
                                    int32_t W, int32_t cin, int32_t cout, int32_t r, int32_t s, int32_t stride,
                                    int32_t pad, void* stream);
int dsp_conv_backward_weight_static_bytes(size_t* bytes);

/* ---- in-situ kernel timing (measurement support) ------------------------------------------------ */

/*
 * Between dsp_profile_start and dsp_profile_stop every kernel launch of the library carries its own
 * start and stop event, filled from the timestamps of that kernel's dispatch on the stream it runs on
 * (at most max_launches launches; events are created here, so call it outside timed regions; not
 * usable under stream capture).  dsp_profile_stop synchronises the device and sums, per
 * kernel name, the launches, the milliseconds between the event pairs and the algorithmic work of
 * the launches: unit_kind 0 = floating-point operations (2 per multiply-accumulate of the
 * convolution as defined, padding taps and skipped strided taps not counted), unit_kind 1 = bytes
 * that have to cross HBM once (each operand read once, each result written once).
 * dsp_profile_get returns entry i of that table.  Process-wide, not thread-safe.
 * dsp_profile_start and dsp_profile_stop each synchronise the device and launch one empty marker kernel
 * (dsp_profile_window_begin / dsp_profile_window_end), so that an external kernel trace of the process can be
 * cut to exactly the launches the table covers.
 */
int dsp_profile_start(int32_t max_launches);
int dsp_profile_stop(int32_t* n_kernels);
int dsp_profile_get(int32_t i, char* name, size_t name_len, int64_t* launches, double* total_ms, double* total_units,
                    int32_t* unit_kind);

const char* dsp_strerror(int status);
/* Text of the most recent failure on this thread ("" if none). */
const char* dsp_last_error(void);
/* Identifies the sources this binary was built from (a hash over csrc/ and this header, set by the build
 * script); the Python binding refuses to load a binary whose id differs from the sources next to it. */
const char* dsp_build_id(void);

#ifdef __cplusplus
}
#endif
#endif /* DSP_H */
