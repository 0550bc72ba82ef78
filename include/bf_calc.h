/*
 * libbf — the paper's analytical model as callable functions (pure host arithmetic, no device).
 *
 * "Breadth-First Pipeline Parallelism" (arXiv 2211.05953) argues with a small model of training
 * efficiency as a function of the batch size per GPU beta = B / N_gpu (Sec. 3, Sec. 4.2, Fig. 2,
 * Table 4.1) and of training cost against time (Sec. 3.5).  These functions evaluate that model.
 *
 * A configuration has N_DP x N_PP x N_TP GPUs, N_mb sequential micro-batches of S_mb samples per
 * data-parallel rank and N_loop stages per pipeline rank, so beta = N_mb S_mb / (N_PP N_TP).
 * beta_net is the constant of Eq. ddp_efficiency: the ratio of gradient-reduction time to
 * computation time is beta_net / (N_mb S_mb) for plain data parallelism (App. A.3.1:
 * beta_net = I_hw / S_seq).
 *
 * All functions are thread-safe and allocate nothing.  Errors: BF_EINVAL (and a text in
 * bf_last_error()) for a configuration the method does not allow.
 */
#ifndef BF_CALC_H
#define BF_CALC_H

#include "bf.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Rows of Table 4.1 that the efficiency model covers. */
typedef enum {
  BF_METHOD_NO_PIPELINE = 0, /* data (and tensor) parallelism with gradient accumulation; N_PP must be 1 */
  BF_METHOD_NON_LOOPED = 1,  /* GPipe / 1F1B: same bubble, network volume and overlap; N_loop must be 1 */
  BF_METHOD_DEPTH_FIRST = 2, /* looped, sequences of N_PP micro-batches; N_mb % N_PP == 0 */
  BF_METHOD_BREADTH_FIRST = 3
} bf_method;

typedef struct {
  int32_t method;   /* bf_method */
  int32_t N_PP, N_loop, N_TP;
  int32_t N_layers; /* > 0: the overlap loses the share N_PP / N_layers of the backward pass that runs after the
                       last gradient is complete (Table 4.1, column "DP overlap"); 0: that share is neglected,
                       as in Eq. ddp_efficiency, Eq. pipeline_efficiency, Eq. pipeline_efficiency_bf */
  int32_t N_mb, S_mb;
  int32_t sharded;  /* 1: fully sharded data parallelism: 3/2 of the network volume, repeated per micro-batch
                       (no pipeline, non-looped), per sequence of N_PP micro-batches (depth-first) or not at
                       all (breadth-first) (Sec. 3.1, Sec. 4.2, App. A.3.1) */
  int32_t overlap;  /* 1: network operations run beside the computation they can overlap with (Eq. efficiency,
                       first branch); 0: nothing is overlapped (second branch, Fig. 2b) */
  double beta_net;
} bf_calc_config;

typedef struct {
  double beta;        /* batch size per GPU, N_mb S_mb / (N_PP N_TP) */
  double bubble;      /* Eq. bubble / Eq. bubble_looped: (N_PP - 1) / (N_mb N_loop) */
  double net_ratio;   /* data-parallel network time / computation time */
  double overlap_share; /* share of the computation the network time can hide under (0 with overlap = 0) */
  double net_overhead;  /* max(0, net_ratio - overlap_share) */
  double efficiency;  /* 1 / (1 + bubble + net_overhead) */
} bf_calc_point;

/* Evaluates the model for one configuration.  BF_EINVAL: sizes < 1, N_mb < N_PP, a depth-first
 * N_mb that is not a multiple of N_PP, N_PP != 1 without a pipeline, N_loop != 1 non-looped,
 * N_layers not a multiple of N_PP N_loop (when given), beta_net < 0. */
bf_status bf_calc_efficiency(const bf_calc_config* cfg, bf_calc_point* out);

/* The curve of Fig. 2: cfg evaluated at N_mb = n_mb[i] for i < n (cfg->N_mb is ignored), S_mb fixed;
 * out[i].efficiency = -1 where the method does not allow that N_mb.  Returns BF_EINVAL only for a
 * null pointer or a cfg that no N_mb makes valid. */
bf_status bf_calc_efficiency_curve(const bf_calc_config* cfg, const int32_t* n_mb, size_t n, bf_calc_point* out);

/* Smallest batch size per GPU at which the data-parallel network time is fully hidden
 * (overlap = 1; the right-hand sides of Eq. ddp_efficiency, Eq. pipeline_efficiency_3d and
 * Eq. pipeline_efficiency_bf, with the factor 3/2 when sharded), for a given N_mb where the bound depends on it. */
bf_status bf_calc_beta_threshold(const bf_calc_config* cfg, double* beta_out);

/* Sec. 3.5.  Eq. critical_batch: samples needed grow as 1 + B / B_crit.  Eq. time_cost_tradeoff at a
 * fixed batch size per GPU beta and utilisation `efficiency` (1 for the equation as printed):
 * cost = (1 + beta N_gpu / B_crit) / efficiency, time = cost / N_gpu, both up to a common factor. */
bf_status bf_calc_cost_time(double beta, double N_gpu, double B_crit, double efficiency, double* cost, double* time);

#ifdef __cplusplus
}
#endif
#endif /* BF_CALC_H */
