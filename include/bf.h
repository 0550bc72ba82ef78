/*
 * libbf — one pipeline rank's training step in breadth-first or depth-first order,
 * on one MI355X (gfx950).
 *
 * Method: "Breadth-First Pipeline Parallelism" (arXiv 2211.05953).  A rank holds
 * N_loop looped stages (Sec. 4.1, N_loop = N_stage / N_PP), each a contiguous chunk
 * of identical transformer layers (App. A.1), and pushes N_mb micro-batches of size
 * S_mb through them.  On one device the stages are chained, which is the N_PP = 1
 * case of the method (App. C, breadth-first gradient accumulation).
 *
 *   BF: every micro-batch through a stage before the next stage (forward-first);
 *       a stage's gradient is final after its N_mb backwards and its fused Adam
 *       step runs there, overlapped with the backward of the earlier stages.
 *   DF: each micro-batch through the whole forward and backward before the next
 *       (App. C); gradients are final only in the last micro-batch's backward.
 *
 * All pointers named "device" are HIP device pointers on the current device, all
 * pointers named "host" are ordinary host memory.  The library never allocates
 * device memory: the caller hands it one workspace of bf_workspace_bytes().  No
 * call throws or aborts; every call returns a bf_status and bf_last_error() gives
 * the reason for the last failure on the calling thread.
 */
#ifndef BF_H
#define BF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct bf_stack bf_stack; /* opaque; owned by the library, lives in host memory */

typedef enum { BF_OK = 0, BF_EINVAL = -1, BF_ENOMEM = -2, BF_ESTATE = -3, BF_EDEVICE = -4 } bf_status;
typedef enum { BF_SCHED_BF = 0, BF_SCHED_DF = 1 } bf_schedule;
/* BF_BF16: bf16 weights and activations in HBM, fp32 accumulators, fp32 master weights,
 * fp32 main-grads, fp32 Adam (mixed precision, App. A.1).  BF_FP32: everything fp32. */
typedef enum { BF_FP32 = 0, BF_BF16 = 1 } bf_dtype;
/* BF_CKPT_LAYER keeps one activation checkpoint (the layer input) per layer and
 * micro-batch and recomputes the layer's forward before its backward (App. A.2.2,
 * Eq. mem_ckpt).  BF_CKPT_NONE keeps every activation the backward needs. */
typedef enum { BF_CKPT_NONE = 0, BF_CKPT_LAYER = 1 } bf_ckpt;
/* Kernel family.  BF_KERNELS_AUTO picks the MFMA kernels wherever the shape allows in
 * bf16 mode; BF_KERNELS_PLAIN forces the simple fp32-FMA kernels (any shape, slow). */
typedef enum { BF_KERNELS_AUTO = 0, BF_KERNELS_PLAIN = 1 } bf_kernels;

/* Parameter tensors of one layer (App. A.1: attention + two-layer MLP).  Row-major.
 * W_QKV columns are [Q | K | V]; head a owns columns a*S_head .. (a+1)*S_head-1 of
 * each third.  y = x W + b for every linear. */
typedef enum {
  BF_LN1_G = 0, BF_LN1_B = 1,
  BF_W_QKV = 2, /* [S_hidden, 3 S_hidden] */ BF_B_QKV = 3,
  BF_W_O = 4,   /* [S_hidden, S_hidden]   */ BF_B_O = 5,
  BF_LN2_G = 6, BF_LN2_B = 7,
  BF_W_FC1 = 8, /* [S_hidden, S_mlp]      */ BF_B_FC1 = 9,
  BF_W_FC2 = 10,/* [S_mlp, S_hidden]      */ BF_B_FC2 = 11,
  BF_N_TENSORS = 12,
  /* Input and output layers (config S_voc > 0; App. A.1), held once, addressed as pseudo-layer N_layers:
   * token embedding [S_voc, S_hidden], position embedding [S_seq, S_hidden], final LayerNorm gain and
   * bias, output projection [S_voc, S_hidden] (not tied to the token embedding). */
  BF_E_TOK = 12, BF_E_POS = 13, BF_LNF_G = 14, BF_LNF_B = 15, BF_W_OUT = 16,
  BF_N_VOCAB_TENSORS = 5
} bf_tensor_id;

typedef struct {
  int32_t S_hidden, N_heads, S_head, S_mlp, S_seq; /* N_heads * S_head == S_hidden */
  int32_t N_layers;                                /* layers held by this rank */
  int32_t N_mb_max, S_mb_max;                      /* size the pre-allocated arena (App. D.2) */
  int32_t dtype;                                   /* bf_dtype */
  int32_t ckpt_mode;                               /* bf_ckpt */
  int32_t causal;                                  /* 1: mask j > i (GPT); 0: bidirectional */
  int32_t kernels;                                 /* bf_kernels */
  int32_t queue_depth;  /* > 0: the host never runs more than this many stage-level ops ahead of
                           the device (App. D.2, bounded kernel queue); 0: unbounded */
  int32_t fuse_wgrad;   /* 1: in breadth-first order the weight-matrix gradients of a stage are taken once per
                           stage, as one product over all its micro-batches, after the stage's last backward
                           (breadth-first groups the work by stage, Sec. 4.2): the fp32 main-grad is written once
                           instead of read-modified-written N_mb times.  The sum over micro-batches is then
                           one long fp32 contraction, so BF and DF gradients agree to rounding, not bitwise.
                           The per-micro-batch operands of one stage are kept until then (with
                           BF_CKPT_LAYER: the recomputed ones).  0: accumulate per micro-batch. */
  int32_t N_loop_min;   /* smallest N_loop bf_run_step will be called with (0 or 1: any).  Sizes the per-stage
                           buffers of fuse_wgrad for ceil(N_layers / N_loop_min) layers; a step whose stages
                           are larger than that accumulates per micro-batch instead. */
  int32_t dp_fs;        /* 1 (bf16 only): fully sharded data parallelism as one GPU can show it (Sec. 3.1, App. D.1).
                           The low-precision weights are not kept resident: the stack holds a double buffer of two
                           stages (each ceil(N_layers / N_loop_min) layers) and reconstructs a stage's bf16 weights
                           from the fp32 master copy (the rank's shard; with one rank, all of it) into the idle
                           half before the stage is used, on the side stream, while the other half computes.
                           A stage still resident in a half is not reconstructed again.  Results are bit-identical
                           to dp_fs = 0; bf_step_report counts the reconstructions (breadth-first: one forward and
                           one backward interval per stage; depth-first: as many per micro-batch, Sec. 4.2).
                           Stages larger than a half: BF_EINVAL from bf_run_step. */
  int32_t S_voc;        /* > 0: the stack also holds the input layer (token + position embedding, attached to
                           the first stage) and the output layer (final LayerNorm, projection to S_voc logits,
                           mean cross-entropy; attached to the last stage), for bf_run_lm_step.  With dp_fs
                           these two keep a resident bf16 copy.  0: none. */
  uint64_t seed;        /* device-side initialisation: weights ~ N(0, init_std), biases 0, LN gain 1 */
  float init_std;
  float ln_eps;
  float lr, beta1, beta2, adam_eps, weight_decay;  /* Adam, bias-corrected, decoupled decay */
  int32_t mb_chains;    /* 2: a breadth-first step runs two micro-batches of a stage side by side.  In breadth-first
                           order every micro-batch of a stage is there before the stage starts and none depends on
                           another (Sec. 4.1), which depth-first order, with one micro-batch in flight, cannot offer:
                           even micro-batches run on the caller's stream, odd ones on a second stream of the stack's,
                           each chain with its own backward temporaries; the chains meet once per stage, for the
                           stage-wide weight-gradient products and the optimizer step.  Pays where one micro-batch's
                           kernels do not fill the chip (a 2048-wide model: step 44 -> 37 ms); costs an 8192-wide one
                           2 to 7 %.  The workspace grows by a second set of backward temporaries and a second fp32
                           gradient arena of the layers' size (with BF_CKPT_LAYER also by a second recomputation
                           record).  Needs fuse_wgrad = 1, dp_fs = 0, queue_depth = 0, S_voc = 0, and y and
                           dx given to bf_run_step / bf_run_rank_step; depth-first steps and steps of
                           one micro-batch run as with 1.  A two-chain step splits no contraction (the one-chain step
                           does where a product has few tiles; results then differ by the rounding of the outputs,
                           otherwise outputs and weight-matrix gradients are the same bits).  Bias and LayerNorm
                           gradients are then (sum over even) + (sum over odd micro-batches): equal to the one-chain
                           result to fp32 rounding, and the same bits from run to run.  0 or 1: one micro-batch at
                           a time. */
} bf_config;

/* Integer event trace of a step. op: 0 forward, 1 backward, 2 optimizer (mb = -1).
 * live_ckpt: activation checkpoints (one per layer and micro-batch) alive after the
 * event, the count of Eq. mem_ckpt. */
typedef struct { int32_t op, stage, mb, live_ckpt; } bf_event;

/* Kernel classes of the per-launch timing (bf_run_step with timing == 2 or 3). */
typedef enum {
  BF_K_GEMM_FWD = 0,   /* Y = X W           (QKV, out-proj, FC1, FC2) */
  BF_K_GEMM_DGRAD = 1, /* dX = dY W^T */
  BF_K_GEMM_WGRAD = 2, /* G += X^T dY into the fp32 main-grad */
  BF_K_ATTN_FWD = 3, BF_K_ATTN_BWD = 4,
  BF_K_LN_FWD = 5, BF_K_LN_BWD = 6, BF_K_COLSUM = 7, BF_K_ADAM = 8,
  BF_K_RECONSTRUCT = 9, /* dp_fs: fp32 master -> bf16 stage weights into a half of the double buffer */
  BF_K_VOCAB = 10,      /* embedding forward / backward and softmax cross-entropy (bf_run_lm_step) */
  BF_N_KERNEL_CLASSES = 11
} bf_kernel_class;

typedef struct {
  double gpu_ms;            /* whole step on the device (events on the caller's stream) */
  double adam_ms;           /* sum of the fused Adam launches */
  double flops_model;       /* 3 x forward (linears + full attention), per step */
  double flops_paper;       /* Eq. compute x S_seq: 4 x forward */
  double flops_executed;    /* what the kernels ran: causal half, in-kernel recompute, checkpoint recompute */
  int64_t peak_ckpt_count;  /* Eq. mem_ckpt first factor as executed */
  int64_t peak_ckpt_bytes;  /* peak_ckpt_count x bytes of one [S_mb, S_seq, S_hidden] tensor */
  int64_t peak_act_bytes;   /* peak bytes of live stored activations (checkpoints and fused_wgrad_bytes included) */
  int64_t state_bytes;      /* weights, Adam moments, main-grads, low-precision weights */
  int32_t n_events;
  int32_t timed;            /* 1 if gpu_ms / adam_ms are valid (bf_run_step ... timing != 0) */
  /* timing == 2 (every class) or 3 (the weight-gradient products): per kernel class, summed over
   * the step's launches: device time between events recorded around each launch on its stream, launch count, algorithmic flops
   * (2 M N K per product; attention with the causal half; backward attention 2.5 x forward) and
   * algorithmic HBM bytes (every operand read once, every result written once).  With two chains of
   * micro-batches (mb_chains = 2) launches of the two streams overlap, so the classes' times add up to
   * more than the step's. */
  double kernel_ms[BF_N_KERNEL_CLASSES];
  double kernel_flops[BF_N_KERNEL_CLASSES];
  double kernel_bytes[BF_N_KERNEL_CLASSES];
  int64_t kernel_launches[BF_N_KERNEL_CLASSES];
  /* dp_fs = 1 (else 0): contiguous runs of ops on one stage in one direction, each of which needs the
   * stage's weights (the paper's count of reconstructions: 2 N_loop breadth-first, 2 N_loop N_mb
   * depth-first at N_PP = 1); reconstructions actually run (a stage found in the double buffer is
   * reused); bytes they moved (4 read + 2 written per parameter); size of the double buffer. */
  int64_t n_weight_intervals;
  int64_t n_reconstruct;
  int64_t reconstruct_bytes;
  int64_t weight_buffer_bytes;
  /* fuse_wgrad = 1 in breadth-first order (else 0): bytes of the per-micro-batch gradients (with
   * BF_CKPT_LAYER also the recomputed operands) of one stage that are kept until the stage's
   * weight-gradient products have run; part of peak_act_bytes. */
  int64_t fused_wgrad_bytes;
  int64_t mb_chains;        /* micro-batch chains the step ran side by side (1 or 2) */
} bf_step_report;

typedef struct {
  int64_t makespan, busy;   /* ticks; busy = N_loop N_mb (t_fwd + t_bwd) */
  int64_t bubble_num, bubble_den; /* (makespan - busy) / busy in lowest terms: Eq. bubble, Eq. bubble_looped */
  int64_t peak_live;        /* peak live (stage, micro-batch) inputs on this rank */
} bf_sched_stats;

/* Bytes of device workspace bf_create_stack needs for cfg; 0 if cfg is invalid. */
size_t bf_workspace_bytes(const bf_config* cfg);

/* Builds a stack inside `workspace` (device, 256-byte aligned, `bytes` long, owned by
 * the caller and kept alive until bf_destroy_stack).  Initialises the parameters on the
 * device from cfg->seed and zeroes the Adam moments.  `stream`: a hipStream_t (NULL =
 * default stream) on which the initialisation is enqueued.
 * BF_EINVAL: bad cfg (N_heads*S_head != S_hidden, sizes < 1, unknown enum ...);
 * BF_ENOMEM: bytes too small; BF_EDEVICE: a HIP call failed. */
bf_status bf_create_stack(const bf_config* cfg, void* workspace, size_t bytes, void* stream, bf_stack** out);
bf_status bf_destroy_stack(bf_stack* s);

/* Number of elements of tensor `tensor_id` of one layer (0 if unknown). */
size_t bf_tensor_elems(const bf_stack* s, int tensor_id);

/* Copy n = bf_tensor_elems fp32 values between host memory and the fp32 master weights
 * (set also refreshes the low-precision copy, or with dp_fs drops what the double buffer
 * holds, and leaves the Adam moments alone).
 * Synchronous.  BF_EINVAL on a bad layer / tensor / n. */
bf_status bf_set_params(bf_stack* s, int layer, int tensor_id, const float* host_src, size_t n);
bf_status bf_get_params(bf_stack* s, int layer, int tensor_id, float* host_dst, size_t n);
/* fp32 main-grads accumulated by the last bf_run_step (sum over its micro-batches,
 * ascending).  BF_ESTATE before the first step. */
bf_status bf_get_grads(bf_stack* s, int layer, int tensor_id, float* host_dst, size_t n);
/* Adam moments: which = 0 first moment, 1 second moment. */
bf_status bf_get_moments(bf_stack* s, int layer, int tensor_id, int which, float* host_dst, size_t n);
/* Zero the Adam moments and reset the step counter to 0.  Synchronous. */
bf_status bf_reset_optimizer(bf_stack* s);

/* One training step of the rank (Sec. 4.1; App. C).
 *   schedule     BF_SCHED_BF or BF_SCHED_DF
 *   N_loop       stages; must divide N_layers
 *   N_mb, S_mb   1..N_mb_max, 1..S_mb_max
 *   x            device, [N_mb, S_mb, S_seq, S_hidden] in the stack's dtype (bf16 or fp32): stage-0 input
 *   dy           device, same shape/dtype: gradient of the loss w.r.t. the last stage's output
 *   y, dx        device outputs, same shape/dtype; either may be NULL
 *   apply_optimizer  0: gradients only; 1: fused Adam per stage when its gradient is final
 *   timing       0: no events; 1: fill report->gpu_ms / adam_ms (synchronises at the end);
 *                2: as 1, plus an event pair around every kernel launch -> report->kernel_*;
 *                3: as 1, plus event pairs around the weight-gradient products only (the class with
 *                   the most time): a few dozen to a few hundred events per step instead of thousands
 *   stream       hipStream_t of the caller (NULL = default stream).  The call is asynchronous
 *                on it (unless timing != 0); the library's own streams (dp_fs reconstructions; the
 *                second chain of cfg.mb_chains = 2) start after what the stream holds at the call and
 *                join it before the call returns, so that later work on the stream comes after the
 *                whole step.  The optimizer runs on the caller's stream (with two chains: on the
 *                stream of the stage's last micro-batch).
 *   report       may be NULL
 * With timing = 0 and cfg.queue_depth = 0 the call enqueues kernel launches and event record / wait
 * only (no allocation, no memset or copy, no host synchronisation) and may be recorded into a HIP
 * graph by stream capture; the optimizer's step count is kept on the device and advanced by the step
 * itself, so replays are successive steps.  The host-side trace and report describe the recorded call.
 * Main-grads stay readable until the next step starts.  x, dy, y, dx must not alias the workspace.
 * BF_EINVAL: N_layers % N_loop != 0, sizes out of range, null x / dy, unknown schedule. */
bf_status bf_run_step(bf_stack* s, int schedule, int N_loop, int N_mb, int S_mb,
                      const void* x, const void* dy, void* y, void* dx,
                      int apply_optimizer, int timing, void* stream, bf_step_report* report);

/* The same step as rank `rank` (0..N_PP-1) of an N_PP-deep looped pipeline runs it (Sec. 4.1, Sec. 4.2): the
 * rank holds the global stages l * N_PP + rank, l = 0..N_loop-1 (N_layers / N_loop layers each), and walks them
 * in the breadth-first order (forward-first, every micro-batch through a stage before the next stage; needs
 * N_mb >= N_PP) or the depth-first order (backward-first, sequences of N_PP micro-batches, interleaved warm-up;
 * needs N_mb % N_PP == 0).  The neighbouring ranks are not run: the caller's buffers stand in for what they
 * would send and receive,
 *   x, dy   device, [N_loop, N_mb, S_mb, S_seq, S_hidden]: input of local stage l for micro-batch m, and the
 *           gradient arriving at that stage's output
 *   y, dx   device outputs of the same shape (either may be NULL): the stage's output and the gradient
 *           leaving its input
 * so the rank's stages do not feed each other (at N_PP = 1 bf_run_step chains them instead).  Everything
 * else (optimizer per stage when its gradient is final, fuse_wgrad in breadth-first order, dp_fs, timing,
 * report, trace with GLOBAL stage indices, error codes) is as for bf_run_step; BF_EINVAL also for a rank
 * outside 0..N_PP-1 or an N_mb the order does not allow. */
bf_status bf_run_rank_step(bf_stack* s, int schedule, int N_PP, int rank, int N_loop, int N_mb, int S_mb,
                           const void* x, const void* dy, void* y, void* dx,
                           int apply_optimizer, int timing, void* stream, bf_step_report* report);

/* The step of bf_run_step on token ids (config S_voc > 0): the input layer feeds the first stage, the output
 * layer and the loss follow the last (App. A.1; the S_voc / (16 N_layers) term of Eq. compute).
 *   tokens, labels   device int32 [N_mb, S_mb, S_seq], ids in 0..S_voc-1.  A token id outside that range
 *                    embeds as the position row alone and gets no gradient; a label outside it leaves its
 *                    position out of the loss.
 *   loss             device float [N_mb]: micro-batch m's share, sum of its tokens' cross-entropies divided by
 *                    N_mb * S_mb * S_seq; the batch loss is the sum of the N_mb entries.
 * A micro-batch's loss and the gradient of the output layer are taken when it leaves the last stage's
 * forward; the input layer's gradient after the first stage's backward, without atomics (every sum in a
 * fixed order).  With apply_optimizer the input layer steps with the first stage and the output layer with
 * the last.  report->flops_* include the output projection.  Other arguments and errors as bf_run_step;
 * BF_ESTATE if the stack was created with S_voc = 0. */
bf_status bf_run_lm_step(bf_stack* s, int schedule, int N_loop, int N_mb, int S_mb,
                         const int32_t* tokens, const int32_t* labels, float* loss,
                         int apply_optimizer, int timing, void* stream, bf_step_report* report);

/* Integer event trace of the last bf_run_step / bf_run_rank_step: copies min(cap, n) events, *n = total. */
bf_status bf_get_trace(const bf_stack* s, bf_event* dst, size_t cap, size_t* n);

/* Pure host arithmetic, no device needed: the order in which rank `rank` of an N_PP-deep
 * looped pipeline runs its ops (stage index in the trace is the GLOBAL stage
 * l*N_PP + rank) and a unit-time simulation of all ranks (forward t_fwd ticks, backward
 * t_bwd, transfers free) giving the bubble of Eq. bubble / Eq. bubble_looped.
 * BF needs N_mb >= N_PP; DF needs N_mb % N_PP == 0 (Sec. 4.1).  No optimizer events.
 * dst may be NULL (cap 0) to query *n. */
bf_status bf_schedule_trace(int schedule, int N_PP, int N_loop, int N_mb, int rank,
                            int t_fwd, int t_bwd, bf_event* dst, size_t cap, size_t* n,
                            bf_sched_stats* stats);

/* Exact parameter count of the stack (biases and LayerNorms included). */
int64_t bf_param_count(const bf_config* cfg);

/* Reason for the last failure on this thread ("" if none). */
const char* bf_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* BF_H */
