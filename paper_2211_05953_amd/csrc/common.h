// Shared declarations of the HIP path: element types, launch helpers, error plumbing.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/bf.h"

namespace bf {

typedef __bf16 bf16_t;

// GEMM operand layouts (all row-major storage):
//   NN  A[M,K]            B[K,N]   forward  Y = X W
//   NT  A[M,K]            B as [N,K]  dgrad  dX = dY W^T
//   TN  A as [K,M]        B[K,N]   wgrad   G = X^T dY   (fp32 output, optional accumulate)
enum Layout { L_NN = 0, L_NT = 1, L_TN = 2 };

// What is done to the fp32 accumulator before it is stored.
enum Epilogue {
  E_NONE = 0,       // C = acc
  E_BIAS = 1,       // C = acc + bias[n]
  E_BIAS_RES = 2,   // C = acc + bias[n] + R[m,n]
  E_BIAS_GELU = 3,  // C = acc + bias[n];  C2 = gelu(C)
  E_GELU_BWD = 4,   // C = acc * gelu'(R[m,n])      (R holds the pre-activation)
  E_ACCUM = 5       // fp32 C = (accumulate ? C : 0) + acc
};

struct GemmArgs {
  int M, N, K;
  const void* A;
  const void* B;
  void* C;
  const float* bias;  // [N] fp32 or null
  const void* R;      // [M,N] in the activation dtype or null
  void* C2;           // second output of E_BIAS_GELU
  int accumulate;     // E_ACCUM only
  // Weight-gradient layout only: the contraction runs over n_seg segments of K rows each, segment i
  // reading A + i * seg_stride_a and B + i * seg_stride_b (elements): one product over all the
  // micro-batches of a stage.  n_seg <= 1 means a single segment.
  int n_seg = 1;
  size_t seg_stride_a = 0, seg_stride_b = 0;
  // Weight-gradient layout only: when not null, the column sums of B over all K rows of all
  // segments (the bias gradient that goes with the weight gradient) are written to colsum[N], fp32,
  // overwritten or added to as `accumulate` says.
  float* colsum = nullptr;
  // Other layouts, epilogue E_GELU_BWD: colsum[N] receives the column sums of the stored output C (the bias
  // gradient of the layer whose pre-activation gradient C is).  With colsum_part, fp32 scratch of
  // ceil(M / 128) * N elements, the MFMA kernel takes them in its epilogue, one row of partial sums per row of
  // tiles, and a small kernel adds the rows up in a fixed order; without it (or on the plain kernel) a second
  // pass over C does.  colsum_rows: set by the MFMA launcher to the rows of partial sums written.
  float* colsum_part = nullptr;
  int* colsum_rows = nullptr;
  // Forward / dgrad layouts with E_ACCUM (matrix-core kernel only): C is [k_slices][M][N] fp32 and slice y of the
  // contraction (K / k_slices long) leaves its partial product in plane y; gemm_splitk_finish adds the planes.
  int k_slices = 1;
  // Forward / dgrad layouts: fp32 scratch for those planes.  With it, gemm() splits the contraction of a product
  // whose tiles would leave half of the chip idle (see gemm_splitk_slices) and finishes it with a second kernel.
  float* splitk_ws = nullptr;
  size_t splitk_ws_elems = 0;
  // The product shares the chip with another stream's kernels (two chains of micro-batches): compute units that
  // its grid leaves idle are taken by those, so nothing is gained by trading a tile's efficiency for a fuller
  // round: no 256 x 192 tile (measured on a 6144-wide stack with two chains: 3066 ms per step without, 3154 with).
  bool shared_chip = false;
};

void set_error(const char* fmt, ...);

#define BF_HIP_CHECK(expr)                                                        \
  do {                                                                            \
    hipError_t e_ = (expr);                                                       \
    if (e_ != hipSuccess) {                                                       \
      bf::set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
      return BF_EDEVICE;                                                          \
    }                                                                             \
  } while (0)

// ---- kernel launchers (each returns BF_OK / BF_EINVAL / BF_EDEVICE) -------------------
// dtype: BF_FP32 or BF_BF16 (activation storage type).
bf_status gemm_plain(int dtype, int layout, int epi, const GemmArgs& a, hipStream_t st);
// true if the MFMA kernel covers this problem (bf16, sizes multiples of its tiles)
bool gemm_mfma_supported(int layout, int epi, int M, int N, int K);
bf_status gemm_mfma(int layout, int epi, const GemmArgs& a, hipStream_t st);
// tile (rows x columns of C per workgroup) the MFMA kernel runs an unsplit product of this shape on; 0 x 0 if none fits
void gemm_mfma_tile(int layout, int epi, int M, int N, int* bm, int* bn);
// Slices the matrix-core path would cut the contraction of this forward / dgrad product into (1: no split).
int gemm_splitk_slices(int layout, int epi, int M, int N, int K);
// C[M,N] (bf16) = epilogue(sum over the planes of part[slices][M][N], added in ascending order); epilogues
// E_NONE, E_BIAS, E_BIAS_RES.
bf_status gemm_splitk_finish(int epi, int M, int N, int slices, const float* part, const float* bias, const void* R,
                             void* C, hipStream_t st);
bf_status gemm(int dtype, int kernels, int layout, int epi, const GemmArgs& a, hipStream_t st);

bf_status layernorm_fwd(int dtype, int T, int h, const void* x, const float* g, const float* b, float eps,
                        void* y, float* stats /*[T][2]: mean, rstd*/, hipStream_t st);
// dx = LN'(dy) (+ dres if non-null);  dg/db (fp32) = or += column sums.
// dcs (may be null): fp32 [h], = or += the column sums of the stored dx (the bias gradient of the linear layer
// that produced x).  part (may be null): fp32 scratch of layernorm_bwd_part_elems(T, h) elements; with it, dx and
// the three column reductions are taken in one pass over dy / x, without it in separate passes.
bf_status layernorm_bwd(int dtype, int T, int h, const void* dy, const void* x, const float* g,
                        const float* stats, const void* dres, void* dx, float* dg, float* db,
                        int accumulate, hipStream_t st, float* dcs = nullptr, float* part = nullptr);
size_t layernorm_bwd_part_elems(int T, int h);
bf_status colsum(int dtype, int T, int N, const void* dY, float* out, int accumulate, hipStream_t st);
// out[n] = (accumulate ? out[n] : 0) + sum_{r < rows} part[r * N + n], rows added in ascending order
bf_status colsum_finish(const float* part, int rows, int N, float* out, int accumulate, hipStream_t st);

bf_status attention_fwd_plain(int dtype, int S_mb, int S_seq, int N_heads, int S_head, int causal,
                              const void* qkv, void* ctx, float* lse, hipStream_t st);
bf_status attention_bwd_plain(int dtype, int S_mb, int S_seq, int N_heads, int S_head, int causal,
                              const void* qkv, const void* ctx, const float* lse, const void* dctx,
                              void* dqkv, float* delta, hipStream_t st);
bool attention_mfma_supported(int S_seq, int S_head);
bf_status attention_fwd_mfma(int S_mb, int S_seq, int N_heads, int S_head, int causal,
                             const void* qkv, void* ctx, float* lse, hipStream_t st);
// part (may be null): the kernels also leave partial column sums of dqkv, attention_bwd_mfma_part_q_rows rows of
// [S_hidden] for dQ (one per sequence and query block) followed by attention_bwd_mfma_part_kv_rows rows of
// [2 S_hidden] for [dK | dV] (one per sequence and block of 128 keys).
bf_status attention_bwd_mfma(int S_mb, int S_seq, int N_heads, int S_head, int causal,
                             const void* qkv, const void* ctx, const float* lse, const void* dctx,
                             void* dqkv, float* delta, hipStream_t st, float* part = nullptr);
size_t attention_bwd_mfma_part_q_rows(int S_mb, int S_seq);
size_t attention_bwd_mfma_part_kv_rows(int S_mb, int S_seq);
bf_status attention_fwd(int dtype, int kernels, int S_mb, int S_seq, int N_heads, int S_head, int causal,
                        const void* qkv, void* ctx, float* lse, hipStream_t st);
// db_qkv (may be null): also db_qkv[3 S_hidden] = (accumulate ? db_qkv : 0) + column sums of dqkv, the bias
// gradient of the QKV projection.  With `part` (attention_bwd_part_elems floats) the matrix-core kernels take the
// sums on their way out and a small kernel adds their partial rows in fixed order; without it, or on the plain
// path, dqkv is read a second time.
bf_status attention_bwd(int dtype, int kernels, int S_mb, int S_seq, int N_heads, int S_head, int causal,
                        const void* qkv, const void* ctx, const float* lse, const void* dctx,
                        void* dqkv, float* delta, hipStream_t st, float* db_qkv = nullptr, float* part = nullptr,
                        int accumulate = 0);
size_t attention_bwd_part_elems(int S_mb, int S_seq, int N_heads, int S_head);
// out[n] = (accumulate ? out[n] : 0) + sum_r pq[r][n] for n < h, + sum_r pkv[r][n - h] for h <= n < 3 h
bf_status attn_bias_finish(const float* pq, int rows_q, const float* pkv, int rows_kv, int h, float* out, int accumulate,
                           hipStream_t st);

// Input layer: x[t, :] = e_tok[tok[t], :] + e_pos[t mod S_seq, :] for n_rows = S_mb * S_seq rows (fp32 tables).
bf_status embedding_fwd(int dtype, int n_rows, int S_seq, int S_voc, int h, const int32_t* tok, const float* e_tok,
                        const float* e_pos, void* x, hipStream_t st);
// g_tok[tok[t], :] += d[t, :] (always added: the caller zeroes g_tok before the first micro-batch);
// g_pos[i, :] = or += sum over the samples of d[b, i, :].
bf_status embedding_bwd(int dtype, int S_mb, int S_seq, int S_voc, int h, const int32_t* tok, const void* d, float* g_tok,
                        float* g_pos, int accumulate_pos, hipStream_t st);
// Softmax cross-entropy of n_rows rows of logits z [n_rows, S_voc] (activation dtype): z is overwritten with
// (softmax(z) - onehot(label)) * scale, row_loss[t] = (logsumexp - z[label]) * scale, loss_out[0] = their sum.
bf_status ce_loss(int dtype, int n_rows, int S_voc, void* z, const int32_t* labels, float scale, float* row_loss,
                  float* loss_out, hipStream_t st);

// Fused Adam over n contiguous parameters; w_lp (bf16 copy) may be null.
// t_dev: device step counter read by the kernel (then t is ignored), or null for the host value t
bf_status adam_step(size_t n, float* w, float* m, float* v, const float* g, bf16_t* w_lp, int t, const int* t_dev, float lr,
                    float beta1, float beta2, float eps, float wd, hipStream_t st);
bf_status bump_step(int* t_dev, hipStream_t st);
bf_status cast_f32_to_bf16(size_t n, const float* src, bf16_t* dst, hipStream_t st);
bf_status fill_f32(size_t n, float* dst, float value, hipStream_t st);
// dst[l * layer_stride + off[k] + i] += src[same] for l < n_layers, k < n_seg <= 8, i < cnt[k]
bf_status add_segments(int n_layers, size_t layer_stride, int n_seg, const size_t* off, const size_t* cnt, float* dst,
                       const float* src, hipStream_t st);
// N(0, std) from a counter-based hash of (seed, index)
bf_status init_normal(size_t n, float* dst, uint64_t seed, float std, hipStream_t st);

}  // namespace bf
