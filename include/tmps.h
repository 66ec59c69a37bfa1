/*
 * tmps.h -- C ABI of libtmps: the stage-training hot path of TiMePReSt
 * (arXiv 2410.14312) on AMD MI355X (gfx950).
 *
 * The paper trains a DNN as a pipeline of W workers, each holding consecutive
 * layers (section "Model Architecture").  A mini-batch of M samples is split
 * into N equal micro-batches; every micro-batch is forwarded on its own, and
 * once the N forwards of a mini-batch are done ONE backward pass is made over
 * the whole mini-batch, differentiating at the weights as they are at that
 * moment (sections "Challenge 1: Staleness of Weights" and "Challenge 2: High
 * Training Time"); the weights are then updated in place (the update rule for
 * TiMePReSt).  Workers order their tasks by nF1B (section "Work Scheduling").
 *
 * Conventions
 *   - Every function returns TMPS_OK (0) or a negative TMPS_E* code unless
 *     stated otherwise; tmps_last_error() gives thread-local text for the last
 *     failure.  Nothing throws or aborts across this boundary.
 *   - "device" pointers are HIP device memory, "host" pointers ordinary
 *     memory.  The caller owns ALL device memory and all streams; the library
 *     allocates only small host structs, freed by tmps_stage_destroy().
 *   - Calls that take a stream are asynchronous on it and never synchronise
 *     the device; tmps_schedule_run() synchronises its streams before it
 *     returns.  A stream argument is a hipStream_t passed as void*.
 *   - Activations are row-major [rows, D] (dense) or channels-last
 *     [rows, H, W, C]; dense weights [Dout, Din]; filters [Cout, R, S, Cin].
 *   - TMPS_F32: activations, gradients, weights fp32.  TMPS_BF16_F32MASTER:
 *     activations and back-propagated gradients bfloat16, fp32 accumulation,
 *     fp32 master weights, momentum and weight gradients, plus a bf16 working
 *     copy of the weights that the contractions read.
 */
#ifndef TMPS_H
#define TMPS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    TMPS_OK = 0,
    TMPS_EINVAL = -1,       /* null pointer, bad enum, non-positive size */
    TMPS_ESHAPE = -2,       /* layer shapes do not chain / operand layout not accepted */
    TMPS_EMICRO = -3,       /* micro-batches of a mini-batch are not equal-sized */
    TMPS_ESLOT = -4,        /* stash slot in use, not filled, or not a whole mini-batch group */
    TMPS_ESTASH = -5,       /* stash too small for the schedule */
    TMPS_EHIP = -6,         /* a HIP call failed */
    TMPS_EUNSUPPORTED = -7, /* layer kind / combination not built */
    TMPS_ECAP = -8          /* output array too small */
};

enum { TMPS_F32 = 0, TMPS_BF16_F32MASTER = 1 };

/* Layer kinds and the meaning of tmps_layer_desc.dims */
enum {
    TMPS_LINEAR = 1,     /* dims = {Din, Dout, skip, rows}; flags TMPS_FLAG_RELU or TMPS_FLAG_GELU.  rows (0 = 1):
                            rows per sample, the layer maps every row [Din] -> [Dout].  skip > 0: the input of the
                            layer `skip` positions before this one (which must be a TMPS_LAYERNORM) is added to the
                            result: a residual connection around the layers in between */
    TMPS_CONV2D = 2,     /* dims = {H, W, Cin, Cout, R, S, stride, pad}; flags TMPS_FLAG_RELU, TMPS_FLAG_SRC(k) */
    TMPS_MAXPOOL = 3,    /* dims = {H, W, C, k, stride, pad}; padded positions never win */
    TMPS_SOFTMAX_CE = 4, /* dims = {classes, rows}; only as the last layer of the last stage, after a plain
                            TMPS_LINEAR with the same rows; labels are int32 [samples, rows]; the loss is the
                            mean over all rows */
    TMPS_LAYERNORM = 5,  /* dims = {D, rows}; per row of D features, eps 1e-5; parameters gain (w) and shift (b) */
    TMPS_ATTENTION = 6,  /* dims = {S, D, heads}; causal multi-head self-attention; input rows [q | k | v] of 3*D
                            features, output [S, D]; scores scaled by 1/sqrt(D/heads) */
    TMPS_EMBEDDING = 7,  /* dims = {vocab, S, D}; first layer of a stage only; the stage input is int32 tokens
                            [samples, S]; output [S, D] = token table row + position table row; parameters
                            token table (w, [vocab, D]) and position table (b, [S, D]) */
    TMPS_AFFINE = 8,     /* dims = {H, W, C}; y = gain[c] * x + shift[c] per channel (channels last), then ReLU with
                            TMPS_FLAG_RELU; parameters gain (w, [C]) and shift (b, [C]); must follow a layer without
                            activation */
    TMPS_RESADD = 9,     /* dims = {H, W, C, k}; y = act(a + b): a = the result of the layer before, b = the result of
                            the layer k positions before (one before the first layer = the stage input);
                            TMPS_FLAG_RELU */
    TMPS_AVGPOOL = 10    /* dims = {H, W, C}; mean over the H*W positions: [H, W, C] -> [C] */
};
enum { TMPS_FLAG_RELU = 1, TMPS_FLAG_GELU = 2 /* exact: z * Phi(z) */ };
/* A convolution normally reads the result of the layer before it.  TMPS_FLAG_SRC(k), k = 2..255, in its flags
 * makes it read the result of the layer k positions before it instead (one position before the first layer of a
 * stage = the stage input): the branch of a residual connection. */
#define TMPS_FLAG_SRC(k) ((int)(k) << 8)

typedef struct tmps_stage tmps_stage; /* opaque */

typedef struct {
    int32_t kind;
    int32_t dims[8];
    int32_t flags;
} tmps_layer_desc;

typedef struct {
    int32_t dtype;        /* TMPS_F32 | TMPS_BF16_F32MASTER */
    int32_t micro_batch;  /* M/N samples per forward */
    int32_t n_micro;      /* N */
    int32_t max_stash;    /* stash capacity in micro-batches; a positive multiple of n_micro */
    int32_t is_last;      /* stage ends in TMPS_SOFTMAX_CE */
    int32_t borrow_input; /* 1: the stage keeps only the pointer x given to tmps_forward_micro,
                             which must stay valid and unchanged until the slot's backward pass,
                             and the N inputs of a mini-batch must be consecutive in memory;
                             0: the input is copied into the stash */
    float lr;             /* learning rate (eta of the update rule) */
    float momentum;       /* mu: buf <- mu*buf + g; w <- w - lr*buf (0 gives the paper's plain SGD) */
} tmps_stage_cfg;

/* ---- stage construction (section "Model Architecture": consecutive layers on one accelerator) ----
 *
 * tmps_stage_bytes: sizes in bytes of the four caller-allocated device regions.
 *   params : [P fp32 master values][P bf16 working copy, TMPS_BF16_F32MASTER only]
 *   state  : [P fp32 momentum][P fp32 weight gradient]
 *   stash  : activations of max_stash micro-batches kept for the backward pass
 *   scratch: gradient ping-pong buffers of one mini-batch and reduction workspace
 * P = tmps_stage_param_count().  All regions must be 256-byte aligned.  Any out pointer may be
 * NULL.  Errors: TMPS_EINVAL, TMPS_ESHAPE (layers do not chain), TMPS_EMICRO, TMPS_EUNSUPPORTED. */
int tmps_stage_bytes(const tmps_layer_desc* layers, int n_layers, const tmps_stage_cfg* cfg,
                     size_t* param_bytes, size_t* state_bytes, size_t* stash_bytes,
                     size_t* scratch_bytes);

/* Create a stage over caller-owned device regions of at least the sizes above.  Touches no
 * device memory: the caller writes the fp32 master parameters (see tmps_stage_param_offset),
 * zeroes `state`, then calls tmps_stage_sync_params().  *out is a host object. */
int tmps_stage_create(tmps_stage** out, const tmps_layer_desc* layers, int n_layers,
                      const tmps_stage_cfg* cfg, void* params, void* state, void* stash,
                      void* scratch);
void tmps_stage_destroy(tmps_stage* stage);

/* Number of trainable scalars P of the stage (weights and biases of all its layers). */
int64_t tmps_stage_param_count(const tmps_stage* stage);
/* Position of a layer's weight (which = 0) or bias (which = 1) inside the flat arrays of P
 * elements (master, working copy, momentum, gradient all use the same order).  A layer without
 * parameters gives count 0. */
int tmps_stage_param_offset(const tmps_stage* stage, int layer, int which, int64_t* offset,
                            int64_t* count);
/* Per-sample element counts of the stage's input and output. */
int64_t tmps_stage_input_elems(const tmps_stage* stage);
int64_t tmps_stage_output_elems(const tmps_stage* stage);
/* Refresh the bf16 working copy from the fp32 master values (no-op for TMPS_F32). */
int tmps_stage_sync_params(tmps_stage* stage, void* hip_stream);
/* Device address inside the stash of the stage output of `slot` (micro_batch x output elements,
 * activation dtype; fp32 logits on the last stage).  Valid until the slot's backward pass; the
 * outputs of the slots of one mini-batch group are consecutive. */
void* tmps_stage_output_ptr(const tmps_stage* stage, int slot);
/* Number of weight updates applied so far (the stage's weight version). */
long tmps_stage_version(const tmps_stage* stage);
/* Stage-wise checkpoints (section "Checkpointing": every stage saves its own parameters after the backward pass of
 * an epoch's last mini-batch, and a run that ended abnormally resumes from the latest epoch all stages completed).
 * The parameters and the optimizer state live in the caller's `params` / `state` regions and are copied by the caller;
 * this call restores the third piece of a stage's state, its update counter (version >= 0; TMPS_EINVAL otherwise, or
 * TMPS_ESLOT while a stash slot is in use: checkpoints are taken between mini-batches).  After writing master
 * parameters into `params`, call tmps_stage_sync_params to refresh the working copy. */
int tmps_stage_set_version(tmps_stage* stage, long version);
/* Graph replay, for stages whose passes are many short kernels (the host then spends longer issuing a pass than the
 * device runs it).  With on != 0, tmps_forward_micro and tmps_backward capture their kernels into a HIP graph the second
 * time they are called with the same device addresses (stash slot, input, upstream gradient, gradient destination, loss
 * destination) and launch that graph from then on; calls with addresses that never repeat keep launching kernel by
 * kernel.  Results are those of the kernel-by-kernel path, bit for bit (the same kernels in the same order).  On the
 * last stage the labels are first copied into the stash (the copy is part of tmps_stage_bytes' stash size), so that
 * the captured loss kernel reads a fixed address; a stage that copies its input (borrow_input = 0) makes that copy
 * outside the graph for the same reason.  While kernel timing is enabled (tmps_profile_enable), and for passes issued on
 * the default stream (which cannot be captured), nothing is captured or replayed.  While a pass is being captured, the
 * runtime refuses to make any other stream wait for an event recorded on the capturing stream (tmps_schedule_run keeps
 * its own threads apart; a caller with threads of its own must do the same around the second call with a set of
 * addresses).  Graphs live with the stage.  Off by default.  Errors: TMPS_EINVAL; a failed capture or instantiation is
 * reported by the pass that attempted it as TMPS_EHIP. */
int tmps_stage_use_graphs(tmps_stage* stage, int on);

/* ---- the three steps of a stage's training step ----
 *
 * Forward pass of one micro-batch (section "Challenge 2", Solution): runs the stage's layers on
 * x (device, micro_batch rows, activation dtype) with the stage's CURRENT weights and keeps in
 * stash slot `slot` (0 <= slot < max_stash) what the backward pass needs.  y (device, may be
 * NULL) receives a copy of the stage output.  On the last stage `labels` (device int32,
 * micro_batch entries) is required, y receives fp32 logits, and loss_out (device float, may be
 * NULL) the mean cross-entropy of the micro-batch.  Errors: TMPS_ESLOT if the slot is in use. */
int tmps_forward_micro(tmps_stage* stage, int slot, const void* x, void* y, const int32_t* labels,
                       float* loss_out, void* hip_stream);

/* For callers that cannot allocate device memory for a workspace -- code under HIP stream capture, tight serving
 * loops, harnesses that forbid hipMalloc: tmps_forward_micro with the fp32 workspace of its contractions (the
 * partial sums of k-split GEMMs, which tmps_forward_micro keeps in the stage's `scratch` region) in a fixed array of
 * TMPS_STATIC_SCRATCH_BYTES that is part of the library's device code; every GPU the library runs on holds one copy
 * of it until the process ends.  Same arguments, results (bit for bit) and errors as tmps_forward_micro; in addition
 * TMPS_ECAP when the stage's forward pass needs a larger workspace (then nothing is launched).  The call allocates
 * nothing, on the device or through any library.  All calls on one GPU share that GPU's array: two calls whose
 * kernels can overlap there (different streams, no dependency between them) race; calls on one stream do not. */
#define TMPS_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
int tmps_forward_micro_static(tmps_stage* stage, int slot, const void* x, void* y, const int32_t* labels,
                              float* loss_out, void* hip_stream);

/* The single backward pass of a mini-batch (section "Challenge 1", Solution): slots must be the
 * n_micro slots g*N .. g*N+N-1 of one group, all filled.  dy (device, M = N*micro_batch rows of
 * the stage output shape, gradient dtype; NULL on the last stage, whose error signal is the
 * gradient of the average of the N micro-batch losses) is propagated through the layers in
 * reverse using the stashed activations and the weights AS THEY ARE NOW; weight gradients are
 * summed over the N micro-batches into `state`; dx (device, M rows of the input shape; may be
 * NULL) receives the gradient w.r.t. the stage input.  Frees the slots, also when the pass fails after its arguments
 * were accepted (TMPS_EUNSUPPORTED, TMPS_EHIP): the gradients are then incomplete and tmps_update must not follow. */
int tmps_backward(tmps_stage* stage, const int* slots, int n_slots, const void* dy, void* dx,
                  void* hip_stream);

/* ---- vertical weight stashing (Methodology, first paragraph; "GPU Memory Overhead") ----
 *
 * The paper keeps every forward pass on one weight version across the workers: a micro-batch is tagged with the
 * number of whole-network updates completed when it enters worker 1, and a later worker, which may have applied newer
 * updates by the time the micro-batch reaches it, runs it on ITS weights after that many updates, which it keeps aside
 * until no forward pass needs them.  Backward passes read the live weights either way.  The calls above implement the
 * in-place reading (every task reads the live weights, nothing is kept); these add the paper's own policy:
 *
 * tmps_stage_set_shadow hands the stage a caller-owned device region (256-byte aligned) for n_versions copies of its
 * `params` region (param_bytes of tmps_stage_bytes each); from then on tmps_update copies the superseded parameters
 * there (one device-to-device copy per update) before it changes them.  n_versions = 0 switches it off.
 * tmps_forward_micro_at is tmps_forward_micro on the weights as they were after `version` updates: the live ones when
 * version is the stage's current version, a kept copy otherwise (TMPS_EINVAL if that version is not kept).
 * tmps_schedule_shadow_versions (host only) tells how many older versions worker `stage` needs under the schedule of
 * W workers and N micro-batches (0 for worker 0, 1 per later worker at W = 4, N = 8).
 * tmps_schedule_run_vsync is tmps_schedule_run with every forward pass on the version it is tagged with (field 6 of
 * the version log, counted from the stages' versions at the start of the run); TMPS_ESTASH if a stage keeps too few. */
int tmps_stage_set_shadow(tmps_stage* stage, void* shadow, size_t bytes, int n_versions);
int tmps_forward_micro_at(tmps_stage* stage, long version, int slot, const void* x, void* y, const int32_t* labels,
                          float* loss_out, void* hip_stream);
int tmps_schedule_shadow_versions(int W, int N, int stage);
int tmps_schedule_run_vsync(tmps_stage** stages, int K, int N, int n_minibatches, const void* inputs,
                            const int32_t* labels, void** hip_streams, float* losses_out,
                            int32_t* version_log_out);

/* ---- the comparison system: PipeDream-style training (related work; the update rule of PipeDream) ----
 *
 * Every batch makes its own forward pass and its own backward pass, workers take them in 1F1B order, and on every
 * worker the backward pass of a batch reads the weights its forward pass read there (horizontal weight stashing); the
 * gradient is applied to the worker's current weights.  Built on the calls above with n_micro = 1 (a batch is a
 * mini-batch of one micro-batch) and on the kept versions of tmps_stage_set_shadow:
 *
 * tmps_backward_at is tmps_backward differentiating at the stage's weights as they were after `version` updates (the
 * live ones when that is the current version, a kept copy otherwise; TMPS_EINVAL if not kept); gradients go to the
 * stage's gradient array as always, and the tmps_update that follows changes the live weights.
 * tmps_schedule_plan_1f1b (host only): the 1F1B task list of W workers for n_batches, 7 int32 per task as
 * tmps_schedule_plan, with micro-batch = -1, field 5 = the number of updates in the weights the task READS and field 6
 * = the number of updates the worker had applied before the task.  Worker s (from 0) has at most W - s batches between
 * their forward and backward pass and reaches back at most W - s - 1 versions.
 * tmps_schedule_run_1f1b runs n_batches that way on K streams: stages[s] created with n_micro = 1, max_stash >= K - s,
 * borrow_input = 1 for s > 0, and a shadow region of at least K - s - 1 versions (TMPS_ESTASH otherwise); inputs,
 * labels, losses_out (one loss per batch) and the log as in tmps_schedule_run, fields 5 and 6 read from the stage
 * objects as the tasks are issued. */
int tmps_backward_at(tmps_stage* stage, long version, const int* slots, int n_slots, const void* dy, void* dx,
                     void* hip_stream);
int tmps_schedule_plan_1f1b(int W, int n_batches, int32_t* ops_out, size_t cap_ops);
int tmps_schedule_run_1f1b(tmps_stage** stages, int K, int n_batches, const void* inputs, const int32_t* labels,
                           void** hip_streams, float* losses_out, int32_t* version_log_out);

/* In-place update (the update rule for TiMePReSt, with momentum): buf <- mu*buf + g,
 * w <- w - lr*buf on the fp32 master values, refreshes the bf16 working copy, version += 1. */
int tmps_update(tmps_stage* stage, void* hip_stream);

/* ---- nF1B schedule (sections "Work Scheduling" and "Multiple Sequence Problem") ----
 *
 * Host-only time-point simulation of W workers, N micro-batches per mini-batch.  Each task is
 * 7 int32: {time-point (from 1), worker (from 0), kind (0 forward, 1 backward+update),
 * mini-batch (from 1), micro-batch (from 0; -1 for a backward), number of updates the worker
 * had applied before the task, whole-network version of the pass the task belongs to}.  The
 * whole-network version counts the mini-batches whose backward pass had left worker 0 before
 * the time-point at which the pass started.  Tasks come in (time-point, worker) order.
 * Returns the number of tasks (also when ops_out is NULL), or TMPS_ECAP / TMPS_EINVAL. */
int tmps_schedule_plan(int W, int N, int n_minibatches, int32_t* ops_out, size_t cap_ops);
/* Mini-batch groups worker `stage` must be able to stash under this schedule. */
int tmps_schedule_stash_groups(int W, int N, int stage);
/* Closed form of the paper for the version difference, floor((W+N-2)/N); TMPS_EINVAL outside
 * its domain W, N >= 2. */
int tmps_version_diff_formula(int W, int N);
/* Steady-state version difference found by simulation. */
int tmps_version_diff_simulated(int W, int N);

/* Run n_minibatches through K stages on K streams of one GPU in nF1B order.  stages[s] must
 * have been created with n_micro = N, borrow_input = 1 for s > 0, and enough stash
 * (tmps_schedule_stash_groups).  inputs: device, n_minibatches*M rows of stage 0's input
 * (int32 tokens when it starts with an embedding); labels: device int32, n_minibatches*M times the rows
 * per sample of the loss layer.  losses_out: device float[n_minibatches], the mean
 * of the N micro-batch losses.  version_log_out: host int32[7 * tasks] as tmps_schedule_plan,
 * except that field 5 is read from the stage objects as the tasks are issued (minus the stage's version when the
 * run started, so that a second run, or a run resumed from a checkpoint, logs the same numbers as the plan); may be NULL.
 * If a task fails, the call still waits for the streams, frees the stash slots of every stage (the mini-batches in
 * flight are lost; updates already applied stay) and returns the first error.
 * Cross-stage dependencies are HIP events.  Each stage's tasks are issued by a host thread of its
 * own (one per stage, joined before the call returns; set the environment variable
 * TMPS_ISSUE_THREADS=0 to issue everything from the calling thread).  The call returns after all K
 * streams are idle. */
int tmps_schedule_run(tmps_stage** stages, int K, int N, int n_minibatches, const void* inputs,
                      const int32_t* labels, void** hip_streams, float* losses_out,
                      int32_t* version_log_out);

/* Streams for tmps_schedule_run.  The runtime spreads streams over a small number of hardware queues in creation
 * order; streams that land on the same queue run one after the other.  tmps_streams_create makes n streams back to
 * back (default priority, non-blocking with respect to the null stream), which puts up to as many of them as there are
 * hardware queues on distinct queues (the runtime uses 4 hardware queues unless the environment variable
 * GPU_MAX_HW_QUEUES, read when HIP starts, says otherwise; K stage streams beside the default stream need K + 1, or two
 * stages take turns on one queue).  out: host array of n stream handles.  The caller destroys them with
 * tmps_streams_destroy once no work is pending on them.  Returns TMPS_OK or TMPS_EHIP. */
int tmps_streams_create(void** out, int n);
int tmps_streams_destroy(void** streams, int n);

/* ---- measurement aid (not part of the method) ----
 *
 * While enabled, every kernel launch made by the calls above is timed with HIP events on the stream
 * it is launched on.  The contraction kernels (the six *_FWD / *_DGRAD / *_WGRAD classes) and the
 * reductions of their k-split (TMPS_KC_SPLIT_FINISH, TMPS_KC_SLICE_SUM) are launched with a start and
 * a stop event of their own, which the runtime stamps with the start and end of that kernel's
 * execution.  The other classes are bracketed by two events recorded around the launch, which also
 * measures dispatch latency; TMPS_KC_EVENT_PAIR is an empty bracket recorded before every update, the
 * cost of such a pair by itself.  tmps_profile_read() waits for the recorded events, adds the elapsed
 * milliseconds and launch counts per class into total_ms[] / launches[] (host arrays of n_classes >=
 * TMPS_KERNEL_CLASSES entries), clears the record and returns TMPS_KERNEL_CLASSES.  Timing adds host
 * overhead: measure throughput with profiling off. */
enum {
    TMPS_KC_DENSE_FWD = 0, TMPS_KC_DENSE_DGRAD, TMPS_KC_DENSE_WGRAD, TMPS_KC_CONV_FWD,
    TMPS_KC_CONV_DGRAD, TMPS_KC_CONV_WGRAD, TMPS_KC_SOFTMAX_CE, TMPS_KC_UPDATE, TMPS_KC_POOL_FWD,
    TMPS_KC_POOL_BWD, TMPS_KC_RELU_MASK, TMPS_KC_REDUCE, TMPS_KC_COPY, TMPS_KC_EVENT_PAIR,
    TMPS_KC_SPLIT_FINISH, TMPS_KC_SLICE_SUM, TMPS_KC_LAYERNORM,
    TMPS_KC_ATTN_FWD, TMPS_KC_ATTN_BWD, TMPS_KC_EMBEDDING, TMPS_KC_AFFINE, TMPS_KC_RESADD, TMPS_KERNEL_CLASSES
};
int tmps_profile_enable(int on);
int tmps_profile_read(double* total_ms, int64_t* launches, int n_classes);

const char* tmps_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* TMPS_H */
