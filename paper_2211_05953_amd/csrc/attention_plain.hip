// Plain attention, forward and backward: one wavefront per query (or key) row, fp32
// arithmetic, scores staged in LDS.  Any head size, S_seq up to 4096, both storage
// types.  It is the fp32-mode attention and the fallback for shapes the MFMA kernels
// do not take.  All reductions run in a fixed order.
//
// Layout: qkv [S_mb, S_seq, 3 S_hidden] packed [Q | K | V], head a at columns
// a*S_head..; ctx [S_mb, S_seq, S_hidden]; lse [S_mb, N_heads, S_seq] = log sum exp of the
// scaled, masked scores of a row.
#include "common.h"

namespace bf {

namespace {

constexpr int ROWS = 4;  // wavefronts (rows) per workgroup

__device__ __forceinline__ float wsum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wmax(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

template <typename T>
__global__ __launch_bounds__(ROWS * 64) void attn_fwd_plain_kernel(const T* __restrict__ qkv, T* __restrict__ ctx,
                                                                   float* __restrict__ lse, int S_seq, int N_heads,
                                                                   int d, int causal, float scale) {
  extern __shared__ float smem[];
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int i = blockIdx.x * ROWS + w;
  const int head = blockIdx.y, b = blockIdx.z;
  const int h = N_heads * d;
  float* sc = smem + (size_t)w * (S_seq + d);
  float* qs = sc + S_seq;
  const bool valid = i < S_seq;  // rows past the end keep running (empty loops) so barriers stay uniform
  const T* base = qkv + (size_t)b * S_seq * 3 * h;
  if (valid) {
    const T* qi = base + (size_t)i * 3 * h + head * d;
    for (int c = lane; c < d; c += 64) qs[c] = (float)qi[c];
  }
  __syncthreads();
  const int jend = !valid ? 0 : (causal ? i + 1 : S_seq);
  float mx = -INFINITY;
  for (int j = lane; j < jend; j += 64) {
    const T* kj = base + (size_t)j * 3 * h + h + head * d;
    float s = 0.f;
    for (int c = 0; c < d; ++c) s = fmaf(qs[c], (float)kj[c], s);
    s *= scale;
    sc[j] = s;
    mx = fmaxf(mx, s);
  }
  mx = wmax(mx);
  float sum = 0.f;
  for (int j = lane; j < jend; j += 64) {
    const float e = expf(sc[j] - mx);
    sc[j] = e;
    sum += e;
  }
  sum = wsum(sum);
  __syncthreads();
  if (!valid) return;
  if (lane == 0) lse[((size_t)b * N_heads + head) * S_seq + i] = mx + logf(sum);
  const float inv = 1.0f / sum;
  for (int c = lane; c < d; c += 64) {
    float acc = 0.f;
    for (int j = 0; j < jend; ++j) acc = fmaf(sc[j], (float)base[(size_t)j * 3 * h + 2 * h + head * d + c], acc);
    ctx[((size_t)b * S_seq + i) * h + head * d + c] = (T)(acc * inv);
  }
}

// delta[b, head, i] = sum_c dctx[i, c] * ctx[i, c]
template <typename T>
__global__ __launch_bounds__(ROWS * 64) void attn_delta_kernel(const T* __restrict__ ctx, const T* __restrict__ dctx,
                                                               float* __restrict__ delta, int S_seq, int N_heads, int d) {
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int i = blockIdx.x * ROWS + w;
  const int head = blockIdx.y, b = blockIdx.z;
  if (i >= S_seq) return;
  const size_t off = ((size_t)b * S_seq + i) * (N_heads * d) + head * d;
  float s = 0.f;
  for (int c = lane; c < d; c += 64) s = fmaf((float)dctx[off + c], (float)ctx[off + c], s);
  s = wsum(s);
  if (lane == 0) delta[((size_t)b * N_heads + head) * S_seq + i] = s;
}

// dq_i = scale * sum_j p_ij (dp_ij - delta_i) k_j
template <typename T>
__global__ __launch_bounds__(ROWS * 64) void attn_bwd_dq_plain_kernel(const T* __restrict__ qkv,
                                                                      const T* __restrict__ dctx,
                                                                      const float* __restrict__ lse,
                                                                      const float* __restrict__ delta,
                                                                      T* __restrict__ dqkv, int S_seq, int N_heads,
                                                                      int d, int causal, float scale) {
  extern __shared__ float smem[];
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int i = blockIdx.x * ROWS + w;
  const int head = blockIdx.y, b = blockIdx.z;
  const int h = N_heads * d;
  float* ds = smem + (size_t)w * (S_seq + 2 * d);
  float* qs = ds + S_seq;
  float* dos = qs + d;
  const bool valid = i < S_seq;
  const T* base = qkv + (size_t)b * S_seq * 3 * h;
  float l = 0.f, dl = 0.f;
  if (valid) {
    const size_t orow = ((size_t)b * S_seq + i) * h + head * d;
    for (int c = lane; c < d; c += 64) {
      qs[c] = (float)base[(size_t)i * 3 * h + head * d + c];
      dos[c] = (float)dctx[orow + c];
    }
    const size_t st = ((size_t)b * N_heads + head) * S_seq + i;
    l = lse[st];
    dl = delta[st];
  }
  __syncthreads();
  const int jend = !valid ? 0 : (causal ? i + 1 : S_seq);
  for (int j = lane; j < jend; j += 64) {
    const T* kj = base + (size_t)j * 3 * h + h + head * d;
    const T* vj = base + (size_t)j * 3 * h + 2 * h + head * d;
    float s = 0.f, dp = 0.f;
    for (int c = 0; c < d; ++c) {
      s = fmaf(qs[c], (float)kj[c], s);
      dp = fmaf(dos[c], (float)vj[c], dp);
    }
    const float p = expf(s * scale - l);
    ds[j] = p * (dp - dl) * scale;
  }
  __syncthreads();
  if (!valid) return;
  for (int c = lane; c < d; c += 64) {
    float acc = 0.f;
    for (int j = 0; j < jend; ++j) acc = fmaf(ds[j], (float)base[(size_t)j * 3 * h + h + head * d + c], acc);
    dqkv[((size_t)b * S_seq + i) * 3 * h + head * d + c] = (T)acc;
  }
}

// dk_j = scale * sum_i p_ij (dp_ij - delta_i) q_i ;  dv_j = sum_i p_ij dctx_i
template <typename T>
__global__ __launch_bounds__(ROWS * 64) void attn_bwd_dkv_plain_kernel(const T* __restrict__ qkv,
                                                                       const T* __restrict__ dctx,
                                                                       const float* __restrict__ lse,
                                                                       const float* __restrict__ delta,
                                                                       T* __restrict__ dqkv, int S_seq, int N_heads,
                                                                       int d, int causal, float scale) {
  extern __shared__ float smem[];
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int j = blockIdx.x * ROWS + w;
  const int head = blockIdx.y, b = blockIdx.z;
  const int h = N_heads * d;
  float* ps = smem + (size_t)w * (2 * S_seq + 2 * d);
  float* ds = ps + S_seq;
  float* ks = ds + S_seq;
  float* vs = ks + d;
  const bool valid = j < S_seq;
  const T* base = qkv + (size_t)b * S_seq * 3 * h;
  if (valid) {
    for (int c = lane; c < d; c += 64) {
      ks[c] = (float)base[(size_t)j * 3 * h + h + head * d + c];
      vs[c] = (float)base[(size_t)j * 3 * h + 2 * h + head * d + c];
    }
  }
  __syncthreads();
  const int ibeg = !valid ? S_seq : (causal ? j : 0);
  const float* lrow = lse + ((size_t)b * N_heads + head) * S_seq;
  const float* drow = delta + ((size_t)b * N_heads + head) * S_seq;
  for (int i = ibeg + lane; i < S_seq; i += 64) {
    const T* qi = base + (size_t)i * 3 * h + head * d;
    const T* doi = dctx + ((size_t)b * S_seq + i) * h + head * d;
    float s = 0.f, dp = 0.f;
    for (int c = 0; c < d; ++c) {
      s = fmaf((float)qi[c], ks[c], s);
      dp = fmaf((float)doi[c], vs[c], dp);
    }
    const float p = expf(s * scale - lrow[i]);
    ps[i] = p;
    ds[i] = p * (dp - drow[i]) * scale;
  }
  __syncthreads();
  if (!valid) return;
  for (int c = lane; c < d; c += 64) {
    float dk = 0.f, dv = 0.f;
    for (int i = ibeg; i < S_seq; ++i) {
      dk = fmaf(ds[i], (float)base[(size_t)i * 3 * h + head * d + c], dk);
      dv = fmaf(ps[i], (float)dctx[((size_t)b * S_seq + i) * h + head * d + c], dv);
    }
    dqkv[((size_t)b * S_seq + j) * 3 * h + h + head * d + c] = (T)dk;
    dqkv[((size_t)b * S_seq + j) * 3 * h + 2 * h + head * d + c] = (T)dv;
  }
}

bool plain_ok(int S_mb, int S_seq, int N_heads, int S_head) {
  if (S_mb < 1 || S_seq < 1 || N_heads < 1 || S_head < 1) { set_error("attention: bad size"); return false; }
  if (S_seq > 4096 || S_head > 512) { set_error("attention (plain kernels): S_seq <= 4096 and S_head <= 512 only"); return false; }
  if (N_heads > 65535 || S_mb > 65535) { set_error("attention: N_heads, S_mb <= 65535"); return false; }
  return true;
}

template <typename K>
bool allow_lds(K kernel, size_t bytes) {
  if (bytes <= 48 * 1024) return true;
  hipError_t e = hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  if (e != hipSuccess) { set_error("attention (plain kernels): cannot reserve %zu bytes of LDS: %s", bytes, hipGetErrorString(e)); return false; }
  return true;
}

template <typename T>
bf_status fwd_t(int S_mb, int S_seq, int N_heads, int d, int causal, const void* qkv, void* ctx, float* lse, hipStream_t st) {
  dim3 grid((S_seq + ROWS - 1) / ROWS, N_heads, S_mb);
  const size_t sh = (size_t)ROWS * (S_seq + d) * sizeof(float);
  if (!allow_lds(attn_fwd_plain_kernel<T>, sh)) return BF_EDEVICE;
  attn_fwd_plain_kernel<T><<<grid, ROWS * 64, sh, st>>>((const T*)qkv, (T*)ctx, lse, S_seq, N_heads, d, causal,
                                                        1.0f / sqrtf((float)d));
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_error("attention_fwd_plain launch failed: %s", hipGetErrorString(e)); return BF_EDEVICE; }
  return BF_OK;
}

template <typename T>
bf_status bwd_t(int S_mb, int S_seq, int N_heads, int d, int causal, const void* qkv, const void* ctx, const float* lse,
                const void* dctx, void* dqkv, float* delta, hipStream_t st) {
  dim3 grid((S_seq + ROWS - 1) / ROWS, N_heads, S_mb);
  const float scale = 1.0f / sqrtf((float)d);
  if (!allow_lds(attn_bwd_dq_plain_kernel<T>, (size_t)ROWS * (S_seq + 2 * d) * sizeof(float))) return BF_EDEVICE;
  if (!allow_lds(attn_bwd_dkv_plain_kernel<T>, (size_t)ROWS * (2 * S_seq + 2 * d) * sizeof(float))) return BF_EDEVICE;
  attn_delta_kernel<T><<<grid, ROWS * 64, 0, st>>>((const T*)ctx, (const T*)dctx, delta, S_seq, N_heads, d);
  attn_bwd_dq_plain_kernel<T><<<grid, ROWS * 64, (size_t)ROWS * (S_seq + 2 * d) * sizeof(float), st>>>(
      (const T*)qkv, (const T*)dctx, lse, delta, (T*)dqkv, S_seq, N_heads, d, causal, scale);
  attn_bwd_dkv_plain_kernel<T><<<grid, ROWS * 64, (size_t)ROWS * (2 * S_seq + 2 * d) * sizeof(float), st>>>(
      (const T*)qkv, (const T*)dctx, lse, delta, (T*)dqkv, S_seq, N_heads, d, causal, scale);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_error("attention_bwd_plain launch failed: %s", hipGetErrorString(e)); return BF_EDEVICE; }
  return BF_OK;
}

}  // namespace

bf_status attention_fwd_plain(int dtype, int S_mb, int S_seq, int N_heads, int S_head, int causal, const void* qkv,
                              void* ctx, float* lse, hipStream_t st) {
  if (!qkv || !ctx || !lse) { set_error("attention_fwd: null pointer"); return BF_EINVAL; }
  if (!plain_ok(S_mb, S_seq, N_heads, S_head)) return BF_EINVAL;
  if (dtype == BF_BF16) return fwd_t<bf16_t>(S_mb, S_seq, N_heads, S_head, causal, qkv, ctx, lse, st);
  return fwd_t<float>(S_mb, S_seq, N_heads, S_head, causal, qkv, ctx, lse, st);
}

bf_status attention_bwd_plain(int dtype, int S_mb, int S_seq, int N_heads, int S_head, int causal, const void* qkv,
                              const void* ctx, const float* lse, const void* dctx, void* dqkv, float* delta,
                              hipStream_t st) {
  if (!qkv || !ctx || !lse || !dctx || !dqkv || !delta) { set_error("attention_bwd: null pointer"); return BF_EINVAL; }
  if (!plain_ok(S_mb, S_seq, N_heads, S_head)) return BF_EINVAL;
  if (dtype == BF_BF16) return bwd_t<bf16_t>(S_mb, S_seq, N_heads, S_head, causal, qkv, ctx, lse, dctx, dqkv, delta, st);
  return bwd_t<float>(S_mb, S_seq, N_heads, S_head, causal, qkv, ctx, lse, dctx, dqkv, delta, st);
}

bf_status attention_fwd(int dtype, int kernels, int S_mb, int S_seq, int N_heads, int S_head, int causal,
                        const void* qkv, void* ctx, float* lse, hipStream_t st) {
  if (dtype == BF_BF16 && kernels == BF_KERNELS_AUTO && attention_mfma_supported(S_seq, S_head)) {
    if (!qkv || !ctx || !lse) { set_error("attention_fwd: null pointer"); return BF_EINVAL; }
    return attention_fwd_mfma(S_mb, S_seq, N_heads, S_head, causal, qkv, ctx, lse, st);
  }
  return attention_fwd_plain(dtype, S_mb, S_seq, N_heads, S_head, causal, qkv, ctx, lse, st);
}

size_t attention_bwd_part_elems(int S_mb, int S_seq, int N_heads, int S_head) {
  if (S_mb < 1 || N_heads < 1 || !attention_mfma_supported(S_seq, S_head)) return 0;
  const size_t h = (size_t)N_heads * S_head;
  return attention_bwd_mfma_part_q_rows(S_mb, S_seq) * h + attention_bwd_mfma_part_kv_rows(S_mb, S_seq) * 2 * h;
}

bf_status attention_bwd(int dtype, int kernels, int S_mb, int S_seq, int N_heads, int S_head, int causal,
                        const void* qkv, const void* ctx, const float* lse, const void* dctx, void* dqkv, float* delta,
                        hipStream_t st, float* db_qkv, float* part, int accumulate) {
  const int h = N_heads * S_head;
  bf_status r;
  if (dtype == BF_BF16 && kernels == BF_KERNELS_AUTO && attention_mfma_supported(S_seq, S_head)) {
    if (!qkv || !ctx || !lse || !dctx || !dqkv || !delta) { set_error("attention_bwd: null pointer"); return BF_EINVAL; }
    float* use = db_qkv ? part : nullptr;
    r = attention_bwd_mfma(S_mb, S_seq, N_heads, S_head, causal, qkv, ctx, lse, dctx, dqkv, delta, st, use);
    if (r != BF_OK || !db_qkv) return r;
    if (use) {
      const size_t rq = attention_bwd_mfma_part_q_rows(S_mb, S_seq), rkv = attention_bwd_mfma_part_kv_rows(S_mb, S_seq);
      return attn_bias_finish(use, (int)rq, use + rq * h, (int)rkv, h, db_qkv, accumulate, st);
    }
  } else {
    r = attention_bwd_plain(dtype, S_mb, S_seq, N_heads, S_head, causal, qkv, ctx, lse, dctx, dqkv, delta, st);
    if (r != BF_OK || !db_qkv) return r;
  }
  return colsum(dtype, S_mb * S_seq, 3 * h, dqkv, db_qkv, accumulate, st);
}

}  // namespace bf
