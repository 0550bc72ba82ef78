/*
 * libbf — the single kernels of the transformer layer (App. A.1 of arXiv 2211.05953:
 * self-attention with N_heads heads of size S_head followed by a two-layer MLP), exported
 * one by one so that each can be checked against the CPU oracle and timed on its own.
 * bf_run_step (bf.h) chains exactly these.
 *
 * All tensor pointers are device pointers; row-major; `dtype` is a bf_dtype and names the
 * storage type of activations and weights (bf16 or fp32; accumulation is always fp32).
 * bias / LayerNorm parameters / statistics / lse / main-grads are fp32.
 * `kernels` is a bf_kernels value.  `stream` is a hipStream_t (NULL = default stream);
 * every call is asynchronous on it.  Nothing is allocated; the caller owns every buffer.
 * Errors: BF_EINVAL for bad sizes / null pointers / unknown enums, BF_EDEVICE if the
 * launch fails; bf_last_error() has the text.
 */
#ifndef BF_OPS_H
#define BF_OPS_H

#include "bf.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Operand layouts of the three linear-layer products (8 flop per parameter and token in
 * total, App. A.1):
 *   BF_NN  forward  C[M,N] = A[M,K] B[K,N]
 *   BF_NT  dgrad    C[M,N] = A[M,K] Bt[N,K]^T          (B passed as [N,K])
 *   BF_TN  wgrad    C[M,N] = At[K,M]^T B[K,N]          (A passed as [K,M]; C is fp32) */
typedef enum { BF_NN = 0, BF_NT = 1, BF_TN = 2 } bf_layout;

/* What happens to the fp32 accumulator acc[m,n] before it is stored:
 *   BF_EPI_NONE       C = acc
 *   BF_EPI_BIAS       C = acc + bias[n]
 *   BF_EPI_BIAS_RES   C = acc + bias[n] + R[m,n]
 *   BF_EPI_BIAS_GELU  C = acc + bias[n] (rounded to dtype), C2 = gelu_tanh(C)
 *   BF_EPI_GELU_BWD   C = acc * gelu_tanh'(R[m,n])
 *   BF_EPI_ACCUM      fp32 C = (accumulate ? C : 0) + acc        (main-grad accumulation) */
typedef enum { BF_EPI_NONE = 0, BF_EPI_BIAS = 1, BF_EPI_BIAS_RES = 2, BF_EPI_BIAS_GELU = 3,
               BF_EPI_GELU_BWD = 4, BF_EPI_ACCUM = 5 } bf_epilogue;

bf_status bf_op_gemm(int dtype, int kernels, int layout, int epilogue, int M, int N, int K,
                     const void* A, const void* B, void* C, const float* bias, const void* R, void* C2,
                     int accumulate, void* stream);
/* The dgrad product in front of a GeLU with the bias gradient of the linear layer below it (App. A.1: the first
 * linear layer of the MLP) taken on the way:
 *   C[M,N] = (A[M,K] Bt[N,K]^T) * gelu_tanh'(R[M,N])            (BF_NT with BF_EPI_GELU_BWD)
 *   db[N]  = (accumulate ? db : 0) + sum_m C[m,:]                of the stored (rounded) C
 * part: device fp32 scratch of ceil(M / 128) * N elements, owned by the caller: with it the MFMA kernel takes the
 * sums in its epilogue (one row of partial sums per row of tiles, added up in a fixed order by a small kernel);
 * NULL, or a problem that goes to the plain kernel: a second pass over C takes them.  db: device fp32 [N]. */
bf_status bf_op_gemm_gelu_bwd_colsum(int dtype, int kernels, int M, int N, int K, const void* A, const void* Bt, void* C,
                                     const void* R, float* db, float* part, int accumulate, void* stream);
/* bf_op_gemm for the forward / dgrad layouts (BF_NN, BF_NT; epilogues none, bias, bias + residual) with scratch for a
 * split contraction: a bf16 product on the matrix cores whose tiles would fill at most half of the chip in its only
 * round, with K >= 2048, runs K in bf_op_gemm_splitk_slices(...) slices on that many times the workgroups; each slice
 * leaves an fp32 plane in `planes` (device, slices * M * N floats, owned by the caller) and a second kernel adds the
 * planes in ascending order and applies the epilogue, so the result does not depend on the order the slices finish
 * in.  Any other shape, dtype or kernel choice, planes == NULL or planes_elems too small: exactly bf_op_gemm. */
bf_status bf_op_gemm_splitk(int dtype, int kernels, int layout, int epilogue, int M, int N, int K, const void* A,
                            const void* B, void* C, const float* bias, const void* R, float* planes,
                            size_t planes_elems, void* stream);
/* Slices that call would use for this shape (1: the contraction is not split). */
int bf_op_gemm_splitk_slices(int layout, int epilogue, int M, int N, int K);
/* 1 if the MFMA kernel takes this problem in bf16 mode, 0 if the plain kernel would run. */
int bf_op_gemm_uses_mfma(int layout, int epilogue, int M, int N, int K);
/* The tile of C (rows x columns per workgroup) that the MFMA kernel runs an unsplit product of this shape on by itself:
 * 256 x 256, 256 x 128, 128 x 128, or 256 x 192 (forward and dgrad layouts with the epilogues none, bias, bias + residual
 * and N a multiple of 192, where that fills the rounds of the grid better: 2048 x 6144 outputs are 256 such tiles).  A
 * step that runs two chains of micro-batches does not take the last shape.  Host arithmetic only.  Returns 1 and the tile in tile_m / tile_n (host ints), or 0
 * (and 0 x 0) where bf_op_gemm_uses_mfma is 0. */
int bf_op_gemm_tile(int layout, int epilogue, int M, int N, int K, int* tile_m, int* tile_n);

/* Weight and bias gradient of one linear layer over all the micro-batches of a stage in one
 * product (breadth-first order: every micro-batch of the stage has been through its backward
 * before the gradient is needed, Sec. 4.2; fp32 main-grads, App. D):
 *   G[M,N]  = (accumulate ? G  : 0) + sum_{i < n_seg} X_i[K,M]^T dY_i[K,N]
 *   db[N]   = (accumulate ? db : 0) + sum_{i < n_seg} sum_k dY_i[k,:]          (db may be NULL)
 * X_i = X + i * stride_x and dY_i = dY + i * stride_dy (strides in elements; the MFMA kernel takes
 * bf16 segments that are 16-byte aligned, others go to the plain kernel), both in the activation dtype, device memory; G and db fp32, device
 * memory, owned by the caller.  BF_EINVAL for bad sizes, null X / dY / G or n_seg < 1. */
bf_status bf_op_wgrad(int dtype, int kernels, int M, int N, int K, int n_seg, const void* X, size_t stride_x,
                      const void* dY, size_t stride_dy, float* G, float* db, int accumulate, void* stream);

/* y = (x - mean) * rstd * g + b per row of x[T,h]; stats[T][2] = (mean, rstd), rstd = 1/sqrt(var + eps). */
bf_status bf_op_layernorm_fwd(int dtype, int T, int h, const void* x, const float* g, const float* b, float eps,
                              void* y, float* stats, void* stream);
/* dx[T,h] = LN'(dy) (+ dres if non-null); dg[h], db[h] (fp32) = or += the column sums. */
bf_status bf_op_layernorm_bwd(int dtype, int T, int h, const void* dy, const void* x, const float* g,
                              const float* stats, const void* dres, void* dx, float* dg, float* db,
                              int accumulate, void* stream);
/* The same with everything a LayerNorm needs in the backward pass taken in one pass over dy and x:
 * dx as above; dg, db as above; dcs[h] (fp32, may be NULL) = or += the column sums of the stored dx, which are the bias
 * gradient of the linear layer that produced x (x = residual + linear output).
 * part: device fp32 scratch of bf_op_layernorm_bwd_part_elems(T, h) elements, owned by the caller: with it (and h a
 * multiple of the vector width, at most 4 x 256 vectors per row) a workgroup walks a run of rows with its column sums in
 * registers and a second small kernel adds the workgroups' partial sums in a fixed order; NULL: separate passes. */
bf_status bf_op_layernorm_bwd_fused(int dtype, int T, int h, const void* dy, const void* x, const float* g,
                                    const float* stats, const void* dres, void* dx, float* dg, float* db, float* dcs,
                                    float* part, int accumulate, void* stream);
size_t bf_op_layernorm_bwd_part_elems(int T, int h);
/* out[N] (fp32) = or += sum over rows of dY[T,N]: the bias gradient. */
bf_status bf_op_colsum(int dtype, int T, int N, const void* dY, float* out, int accumulate, void* stream);

/* Multi-head attention.  qkv [S_mb, S_seq, 3 S_hidden] packed [Q | K | V] with head a at
 * columns a*S_head.. of each third; ctx [S_mb, S_seq, S_hidden]; lse [S_mb, N_heads, S_seq] =
 * log-sum-exp of a row's scaled (1/sqrt(S_head)) and masked scores.  causal = 1 masks j > i. */
bf_status bf_op_attention_fwd(int dtype, int kernels, int S_mb, int S_seq, int N_heads, int S_head, int causal,
                              const void* qkv, void* ctx, float* lse, void* stream);
/* dqkv from dctx; delta is fp32 scratch of S_mb * N_heads * S_seq elements. */
bf_status bf_op_attention_bwd(int dtype, int kernels, int S_mb, int S_seq, int N_heads, int S_head, int causal,
                              const void* qkv, const void* ctx, const float* lse, const void* dctx,
                              void* dqkv, float* delta, void* stream);
/* The same with the bias gradient of the QKV projection (App. A.1: qkv = a W_qkv + b_qkv, so the gradient of b_qkv
 * is the column sum of dqkv over the S_mb * S_seq rows): db_qkv[3 S_hidden] (device fp32) = (accumulate ? db_qkv : 0)
 * + those sums.  part: device fp32 scratch of bf_op_attention_bwd_part_elems(...) elements owned by the caller (0
 * elements: shape not served by the matrix-core kernels); with it the two backward kernels leave per query / key
 * block partial sums of what they store (before rounding to bf16) and one small kernel adds them in a fixed order;
 * NULL, fp32, or a shape outside the matrix-core kernels: dqkv is read a second time (bf_op_colsum). */
bf_status bf_op_attention_bwd_bias(int dtype, int kernels, int S_mb, int S_seq, int N_heads, int S_head, int causal,
                                   const void* qkv, const void* ctx, const float* lse, const void* dctx,
                                   void* dqkv, float* delta, float* db_qkv, float* part, int accumulate, void* stream);
size_t bf_op_attention_bwd_part_elems(int S_mb, int S_seq, int N_heads, int S_head);
/* bf_op_attention_bwd for callers that cannot allocate device memory and have no buffer to lend (code under
 * HIP graph capture, tight serving loops, harnesses that forbid allocation): the same kernels, with `delta` in an
 * array built into the library (BF_ATTENTION_BWD_STATIC_MAX floats = 4 MiB, which every GPU the library runs on
 * holds until the process ends).  Allocates nothing and calls no allocating routine.  BF_EINVAL if
 * S_mb * N_heads * S_seq exceeds the array.  All calls on one GPU share the array: calls that overlap on one GPU
 * (different streams or threads) race; calls on one stream do not.  Nothing in the array has to be cleared
 * between calls (each call writes every element it reads). */
#define BF_ATTENTION_BWD_STATIC_MAX ((size_t)1 << 20)
bf_status bf_op_attention_bwd_static(int dtype, int kernels, int S_mb, int S_seq, int N_heads, int S_head, int causal,
                                     const void* qkv, const void* ctx, const float* lse, const void* dctx,
                                     void* dqkv, void* stream);
int bf_op_attention_uses_mfma(int S_seq, int S_head);

/* Input layer (App. A.1): x[t, :] = e_tok[tokens[t], :] + e_pos[t mod S_seq, :] for n_rows = S_mb * S_seq rows.
 * tokens: device int32 [n_rows]; e_tok [S_voc, S_hidden], e_pos [S_seq, S_hidden] device fp32; x in `dtype`.
 * An id outside 0..S_voc-1 contributes no token row. */
bf_status bf_op_embedding_fwd(int dtype, int n_rows, int S_seq, int S_voc, int S_hidden, const int32_t* tokens,
                              const float* e_tok, const float* e_pos, void* x, void* stream);
/* Its gradient for one micro-batch d [S_mb, S_seq, S_hidden]: g_tok[tokens[t], :] += d[t, :] (always added,
 * ascending t, no atomics); g_pos[i, :] = (accumulate_pos ? g_pos[i, :] : 0) + sum over samples of d[b, i, :]. */
bf_status bf_op_embedding_bwd(int dtype, int S_mb, int S_seq, int S_voc, int S_hidden, const int32_t* tokens,
                              const void* d, float* g_tok, float* g_pos, int accumulate_pos, void* stream);
/* Softmax cross-entropy over rows of logits z [n_rows, S_voc] (`dtype`), in place: z becomes
 * (softmax(z) - onehot(label)) * scale; row_loss[t] = (logsumexp(z[t]) - z[t, label]) * scale (device fp32
 * [n_rows]); loss_out[0] = sum of row_loss in a fixed order.  A label outside 0..S_voc-1 zeroes its row. */
bf_status bf_op_ce_loss(int dtype, int n_rows, int S_voc, void* z, const int32_t* labels, float scale, float* row_loss,
                        float* loss_out, void* stream);

/* Fused Adam over n contiguous fp32 parameters (bias-corrected, decoupled weight decay), step t >= 1;
 * w_lp: bf16 copy of w to refresh, or NULL. */
bf_status bf_op_adam(size_t n, float* w, float* m, float* v, const float* g, void* w_lp, int t,
                     float lr, float beta1, float beta2, float adam_eps, float weight_decay, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* BF_OPS_H */
