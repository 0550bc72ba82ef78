// C-ABI wrappers of the single kernels (include/bf_ops.h).
#include <mutex>

#include "../../include/bf_ops.h"
#include "common.h"

using namespace bf;

static bool dtype_ok(int dtype, int kernels) {
  if (dtype != BF_FP32 && dtype != BF_BF16) { set_error("unknown dtype %d", dtype); return false; }
  if (kernels != BF_KERNELS_AUTO && kernels != BF_KERNELS_PLAIN) { set_error("unknown kernels %d", kernels); return false; }
  return true;
}

// ---- attention backward without a caller-provided scratch buffer ---------------------------
// The per-query term delta = rowsum(dctx * ctx), which the first backward kernel writes and the second
// reads, lives in a file-scope device array instead of an argument.  Every device that loads the
// library holds its own copy of the array at its own address: the address is looked up once per
// device, with that device current, and kept; host code never uses the array's name otherwise.
constexpr size_t STATIC_DELTA_FLOATS = BF_ATTENTION_BWD_STATIC_MAX;  // 4 MiB per device
static __device__ __align__(256) float scratch[STATIC_DELTA_FLOATS];

namespace {

constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mu;
float* g_scratch_ptr[MAX_DEVICES] = {};

bf_status static_delta(float** out) {
  int dev = -1;
  BF_HIP_CHECK(hipGetDevice(&dev));
  if (dev < 0 || dev >= MAX_DEVICES) { set_error("bf_op_attention_bwd_static: device %d outside 0..%d", dev, MAX_DEVICES - 1); return BF_EDEVICE; }
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    BF_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) { set_error("bf_op_attention_bwd_static: the scratch array has no address on device %d", dev); return BF_EDEVICE; }
    g_scratch_ptr[dev] = (float*)p;
  }
  *out = g_scratch_ptr[dev];
  return BF_OK;
}

}  // namespace

extern "C" {

bf_status bf_op_gemm(int dtype, int kernels, int layout, int epilogue, int M, int N, int K, const void* A, const void* B,
                     void* C, const float* bias, const void* R, void* C2, int accumulate, void* stream) {
  if (!dtype_ok(dtype, kernels)) return BF_EINVAL;
  if (epilogue == E_ACCUM && layout != L_TN) { set_error("BF_EPI_ACCUM goes with BF_TN"); return BF_EINVAL; }
  if (epilogue != E_ACCUM && layout == L_TN) { set_error("BF_TN goes with BF_EPI_ACCUM"); return BF_EINVAL; }
  GemmArgs a{M, N, K, A, B, C, bias, R, C2, accumulate};
  return gemm(dtype, kernels, layout, epilogue, a, (hipStream_t)stream);
}

bf_status bf_op_wgrad(int dtype, int kernels, int M, int N, int K, int n_seg, const void* X, size_t stride_x,
                      const void* dY, size_t stride_dy, float* G, float* db, int accumulate, void* stream) {
  if (!dtype_ok(dtype, kernels)) return BF_EINVAL;
  if (n_seg < 1) { set_error("bf_op_wgrad: n_seg must be at least 1"); return BF_EINVAL; }
  GemmArgs a{M, N, K, X, dY, G, nullptr, nullptr, nullptr, accumulate};
  a.n_seg = n_seg;
  a.seg_stride_a = stride_x;
  a.seg_stride_b = stride_dy;
  a.colsum = db;
  return gemm(dtype, kernels, L_TN, E_ACCUM, a, (hipStream_t)stream);
}

bf_status bf_op_gemm_gelu_bwd_colsum(int dtype, int kernels, int M, int N, int K, const void* A, const void* Bt, void* C,
                                     const void* R, float* db, float* part, int accumulate, void* stream) {
  if (!dtype_ok(dtype, kernels)) return BF_EINVAL;
  if (!db) { set_error("bf_op_gemm_gelu_bwd_colsum: db is null"); return BF_EINVAL; }
  GemmArgs a{M, N, K, A, Bt, C, nullptr, R, nullptr, accumulate};
  a.colsum = db;
  a.colsum_part = part;
  return gemm(dtype, kernels, L_NT, E_GELU_BWD, a, (hipStream_t)stream);
}

bf_status bf_op_gemm_splitk(int dtype, int kernels, int layout, int epilogue, int M, int N, int K, const void* A,
                            const void* B, void* C, const float* bias, const void* R, float* planes, size_t planes_elems,
                            void* stream) {
  if (!dtype_ok(dtype, kernels)) return BF_EINVAL;
  if (epilogue == E_ACCUM || layout == L_TN) { set_error("bf_op_gemm_splitk: forward and dgrad layouts only"); return BF_EINVAL; }
  GemmArgs a{M, N, K, A, B, C, bias, R, nullptr, 0};
  a.splitk_ws = planes;
  a.splitk_ws_elems = planes_elems;
  return gemm(dtype, kernels, layout, epilogue, a, (hipStream_t)stream);
}

int bf_op_gemm_splitk_slices(int layout, int epilogue, int M, int N, int K) { return gemm_splitk_slices(layout, epilogue, M, N, K); }

int bf_op_gemm_uses_mfma(int layout, int epilogue, int M, int N, int K) {
  return gemm_mfma_supported(layout, epilogue, M, N, K) ? 1 : 0;
}

int bf_op_gemm_tile(int layout, int epilogue, int M, int N, int K, int* tile_m, int* tile_n) {
  if (!tile_m || !tile_n) return 0;
  *tile_m = *tile_n = 0;
  if (!gemm_mfma_supported(layout, epilogue, M, N, K)) return 0;
  gemm_mfma_tile(layout, epilogue, M, N, tile_m, tile_n);
  return 1;
}

bf_status bf_op_layernorm_fwd(int dtype, int T, int h, const void* x, const float* g, const float* b, float eps, void* y,
                              float* stats, void* stream) {
  if (!dtype_ok(dtype, 0)) return BF_EINVAL;
  return layernorm_fwd(dtype, T, h, x, g, b, eps, y, stats, (hipStream_t)stream);
}

bf_status bf_op_layernorm_bwd(int dtype, int T, int h, const void* dy, const void* x, const float* g, const float* stats,
                              const void* dres, void* dx, float* dg, float* db, int accumulate, void* stream) {
  if (!dtype_ok(dtype, 0)) return BF_EINVAL;
  return layernorm_bwd(dtype, T, h, dy, x, g, stats, dres, dx, dg, db, accumulate, (hipStream_t)stream);
}

bf_status bf_op_layernorm_bwd_fused(int dtype, int T, int h, const void* dy, const void* x, const float* g,
                                    const float* stats, const void* dres, void* dx, float* dg, float* db, float* dcs,
                                    float* part, int accumulate, void* stream) {
  if (!dtype_ok(dtype, 0)) return BF_EINVAL;
  return layernorm_bwd(dtype, T, h, dy, x, g, stats, dres, dx, dg, db, accumulate, (hipStream_t)stream, dcs, part);
}

size_t bf_op_layernorm_bwd_part_elems(int T, int h) { return T > 0 && h > 0 ? layernorm_bwd_part_elems(T, h) : 0; }

bf_status bf_op_colsum(int dtype, int T, int N, const void* dY, float* out, int accumulate, void* stream) {
  if (!dtype_ok(dtype, 0)) return BF_EINVAL;
  return colsum(dtype, T, N, dY, out, accumulate, (hipStream_t)stream);
}

bf_status bf_op_attention_fwd(int dtype, int kernels, int S_mb, int S_seq, int N_heads, int S_head, int causal,
                              const void* qkv, void* ctx, float* lse, void* stream) {
  if (!dtype_ok(dtype, kernels)) return BF_EINVAL;
  return attention_fwd(dtype, kernels, S_mb, S_seq, N_heads, S_head, causal, qkv, ctx, lse, (hipStream_t)stream);
}

bf_status bf_op_attention_bwd(int dtype, int kernels, int S_mb, int S_seq, int N_heads, int S_head, int causal,
                              const void* qkv, const void* ctx, const float* lse, const void* dctx, void* dqkv,
                              float* delta, void* stream) {
  if (!dtype_ok(dtype, kernels)) return BF_EINVAL;
  return attention_bwd(dtype, kernels, S_mb, S_seq, N_heads, S_head, causal, qkv, ctx, lse, dctx, dqkv, delta,
                       (hipStream_t)stream);
}

bf_status bf_op_attention_bwd_bias(int dtype, int kernels, int S_mb, int S_seq, int N_heads, int S_head, int causal,
                                   const void* qkv, const void* ctx, const float* lse, const void* dctx, void* dqkv,
                                   float* delta, float* db_qkv, float* part, int accumulate, void* stream) {
  if (!dtype_ok(dtype, kernels)) return BF_EINVAL;
  if (!db_qkv) { set_error("bf_op_attention_bwd_bias: db_qkv is null"); return BF_EINVAL; }
  return attention_bwd(dtype, kernels, S_mb, S_seq, N_heads, S_head, causal, qkv, ctx, lse, dctx, dqkv, delta,
                       (hipStream_t)stream, db_qkv, part, accumulate);
}

size_t bf_op_attention_bwd_part_elems(int S_mb, int S_seq, int N_heads, int S_head) {
  return attention_bwd_part_elems(S_mb, S_seq, N_heads, S_head);
}

bf_status bf_op_attention_bwd_static(int dtype, int kernels, int S_mb, int S_seq, int N_heads, int S_head, int causal,
                                                const void* qkv, const void* ctx, const float* lse, const void* dctx, void* dqkv,
                                                void* stream) {
  if (!dtype_ok(dtype, kernels)) return BF_EINVAL;
  if (S_mb < 1 || S_seq < 1 || N_heads < 1) { set_error("bf_op_attention_bwd_static: sizes must be >= 1"); return BF_EINVAL; }
  const size_t need = (size_t)S_mb * (size_t)N_heads * (size_t)S_seq;
  if (need > STATIC_DELTA_FLOATS) {
    set_error("bf_op_attention_bwd_static: S_mb * N_heads * S_seq = %zu exceeds the built-in scratch of %zu elements; "
              "use bf_op_attention_bwd with a buffer of the caller's", need, STATIC_DELTA_FLOATS);
    return BF_EINVAL;
  }
  float* delta = nullptr;
  bf_status r = static_delta(&delta);
  if (r != BF_OK) return r;
  // every element the second kernel reads is written by the first in the same call: nothing has to start at zero
  return attention_bwd(dtype, kernels, S_mb, S_seq, N_heads, S_head, causal, qkv, ctx, lse, dctx, dqkv, delta,
                       (hipStream_t)stream);
}

int bf_op_attention_uses_mfma(int S_seq, int S_head) { return attention_mfma_supported(S_seq, S_head) ? 1 : 0; }

bf_status bf_op_embedding_fwd(int dtype, int n_rows, int S_seq, int S_voc, int S_hidden, const int32_t* tokens,
                              const float* e_tok, const float* e_pos, void* x, void* stream) {
  if (!dtype_ok(dtype, 0)) return BF_EINVAL;
  return embedding_fwd(dtype, n_rows, S_seq, S_voc, S_hidden, tokens, e_tok, e_pos, x, (hipStream_t)stream);
}

bf_status bf_op_embedding_bwd(int dtype, int S_mb, int S_seq, int S_voc, int S_hidden, const int32_t* tokens, const void* d,
                              float* g_tok, float* g_pos, int accumulate_pos, void* stream) {
  if (!dtype_ok(dtype, 0)) return BF_EINVAL;
  return embedding_bwd(dtype, S_mb, S_seq, S_voc, S_hidden, tokens, d, g_tok, g_pos, accumulate_pos, (hipStream_t)stream);
}

bf_status bf_op_ce_loss(int dtype, int n_rows, int S_voc, void* z, const int32_t* labels, float scale, float* row_loss,
                        float* loss_out, void* stream) {
  if (!dtype_ok(dtype, 0)) return BF_EINVAL;
  return ce_loss(dtype, n_rows, S_voc, z, labels, scale, row_loss, loss_out, (hipStream_t)stream);
}

bf_status bf_op_adam(size_t n, float* w, float* m, float* v, const float* g, void* w_lp, int t, float lr, float beta1,
                     float beta2, float adam_eps, float weight_decay, void* stream) {
  return adam_step(n, w, m, v, g, (bf16_t*)w_lp, t, nullptr, lr, beta1, beta2, adam_eps, weight_decay, (hipStream_t)stream);
}

}  // extern "C"
