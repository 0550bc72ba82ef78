// Input and output layers of the language model (App. A.1; the S_voc term of Eq. compute):
// token + position embedding forward and backward, softmax cross-entropy with its gradient
// written in place of the logits.  The projections themselves are the GEMM kernels.
// All HBM-bound row kernels: one 256-thread workgroup per token row.  Every sum has a fixed
// order (no atomics), so the gradients do not depend on scheduling.
#include <math.h>

#include "common.h"

namespace bf {

namespace {

constexpr int ROW_THREADS = 256;

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

template <typename T, int VEC>
struct alignas(sizeof(T) * VEC > 16 ? 16 : sizeof(T) * VEC) Vec {
  T v[VEC];
};

template <typename T, int VEC>
__device__ __forceinline__ void load_vec(const T* p, float (&out)[VEC]) {
  typedef Vec<T, VEC> V;
  V t = *reinterpret_cast<const V*>(p);
#pragma unroll
  for (int i = 0; i < VEC; ++i) out[i] = (float)t.v[i];
}

template <typename T, int VEC>
__device__ __forceinline__ void store_vec(T* p, const float (&in)[VEC]) {
  typedef Vec<T, VEC> V;
  V t;
#pragma unroll
  for (int i = 0; i < VEC; ++i) t.v[i] = (T)in[i];
  *reinterpret_cast<V*>(p) = t;
}

// x[t, :] = E_tok[tok[t], :] + E_pos[t mod S_seq, :]; an id outside 0..S_voc-1 contributes no token row.
template <typename T, int VEC>
__global__ __launch_bounds__(ROW_THREADS) void embedding_fwd_kernel(const int32_t* __restrict__ tok,
                                                                    const float* __restrict__ e_tok,
                                                                    const float* __restrict__ e_pos, T* __restrict__ x,
                                                                    int S_seq, int S_voc, int h) {
  const size_t row = blockIdx.x;
  const int v = tok[row];
  const bool valid = v >= 0 && v < S_voc;
  const float* er = e_tok + (size_t)(valid ? v : 0) * h;
  const float* pr = e_pos + (row % (size_t)S_seq) * h;
  T* xr = x + row * (size_t)h;
  for (int c = threadIdx.x * VEC; c < h; c += ROW_THREADS * VEC) {
    float a[VEC], b[VEC];
    load_vec<float, VEC>(er + c, a);
    load_vec<float, VEC>(pr + c, b);
#pragma unroll
    for (int j = 0; j < VEC; ++j) a[j] = (valid ? a[j] : 0.f) + b[j];
    store_vec<T, VEC>(xr + c, a);
  }
}

// Token-embedding gradient without atomics: the workgroup of the first position that uses a token
// sums the rows of every position using it, in ascending position, and adds the sum to that
// token's gradient row; workgroups of later uses leave at once.  Distinct tokens, distinct rows.
// The positions are found by one wavefront (ballot compaction of a window of ids into LDS, in
// order); a thread keeps up to NCH column chunks in registers so the ids are scanned once.
template <typename T, int VEC>
__global__ __launch_bounds__(ROW_THREADS) void embedding_bwd_tok_kernel(const int32_t* __restrict__ tok,
                                                                        const T* __restrict__ d, float* __restrict__ g_tok,
                                                                        int n_rows, int S_voc, int h) {
  constexpr int WIN = 2048, NCH = 8, GROUP = ROW_THREADS * VEC * NCH;
  __shared__ int list[WIN];
  __shared__ int n_list;
  const int t = blockIdx.x;
  const int v = tok[t];
  if (v < 0 || v >= S_voc) return;
  int earlier = 0;
  for (int i = threadIdx.x; i < t; i += ROW_THREADS) earlier |= tok[i] == v;
  if (__syncthreads_or(earlier)) return;
  const int lane = threadIdx.x & 63;
  float* gr = g_tok + (size_t)v * h;
  for (int c0 = 0; c0 < h; c0 += GROUP) {
    float acc[NCH][VEC];
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch)
#pragma unroll
      for (int j = 0; j < VEC; ++j) acc[ch][j] = 0.f;
    for (int w0 = t; w0 < n_rows; w0 += WIN) {
      const int end = w0 + WIN < n_rows ? w0 + WIN : n_rows;
      __syncthreads();  // the list of the previous window has been read
      if (threadIdx.x < 64) {
        int count = 0;
        for (int base = w0; base < end; base += 64) {
          const int i = base + lane;
          const bool hit = i < end && tok[i] == v;
          const unsigned long long mask = __ballot(hit);
          if (hit) list[count + __popcll(mask & ((1ull << lane) - 1ull))] = i;
          count += __popcll(mask);
        }
        if (lane == 0) n_list = count;
      }
      __syncthreads();
      const int n = n_list;
      for (int k = 0; k < n; ++k) {
        const T* dr = d + (size_t)list[k] * h;
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch) {
          const int c = c0 + (ch * ROW_THREADS + (int)threadIdx.x) * VEC;
          if (c < h) {
            float r[VEC];
            load_vec<T, VEC>(dr + c, r);
#pragma unroll
            for (int j = 0; j < VEC; ++j) acc[ch][j] += r[j];
          }
        }
      }
    }
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
      const int c = c0 + (ch * ROW_THREADS + (int)threadIdx.x) * VEC;
      if (c < h) {
        float g[VEC];
        load_vec<float, VEC>(gr + c, g);
#pragma unroll
        for (int j = 0; j < VEC; ++j) g[j] += acc[ch][j];
        store_vec<float, VEC>(gr + c, g);
      }
    }
  }
}

// Position-embedding gradient: position i sums its row over the samples of the micro-batch.
template <typename T, int VEC>
__global__ __launch_bounds__(ROW_THREADS) void embedding_bwd_pos_kernel(const T* __restrict__ d, float* __restrict__ g_pos,
                                                                        int S_mb, int S_seq, int h, int accumulate) {
  const size_t i = blockIdx.x;
  float* gr = g_pos + i * (size_t)h;
  for (int c = threadIdx.x * VEC; c < h; c += ROW_THREADS * VEC) {
    float acc[VEC];
#pragma unroll
    for (int j = 0; j < VEC; ++j) acc[j] = 0.f;
    for (int b = 0; b < S_mb; ++b) {
      float r[VEC];
      load_vec<T, VEC>(d + ((size_t)b * S_seq + i) * h + c, r);
#pragma unroll
      for (int j = 0; j < VEC; ++j) acc[j] += r[j];
    }
    if (accumulate) {
      float g[VEC];
      load_vec<float, VEC>(gr + c, g);
#pragma unroll
      for (int j = 0; j < VEC; ++j) acc[j] += g[j];
    }
    store_vec<float, VEC>(gr + c, acc);
  }
}

// Row-wise softmax cross-entropy.  One pass finds the running maximum and the sum of exponentials
// (rescaled when the maximum moves), a second writes dz = (softmax(z) - onehot(label)) * scale over
// z.  row_loss = (logsumexp(z) - z[label]) * scale.  A label outside 0..S_voc-1 gives a zero row.
template <typename T, int VEC>
__global__ __launch_bounds__(ROW_THREADS) void ce_loss_kernel(T* __restrict__ z, const int32_t* __restrict__ labels,
                                                              float* __restrict__ row_loss, int S_voc, float scale) {
  __shared__ float red_m[4], red_s[4];
  const size_t row = blockIdx.x;
  T* zr = z + row * (size_t)S_voc;
  const int label = labels[row];
  const bool valid = label >= 0 && label < S_voc;
  const float z_label = valid ? (float)zr[label] : 0.f;
  float m = -INFINITY, s = 0.f;
  for (int c = threadIdx.x * VEC; c < S_voc; c += ROW_THREADS * VEC) {
    float v[VEC];
    load_vec<T, VEC>(zr + c, v);
    float cm = v[0];
#pragma unroll
    for (int j = 1; j < VEC; ++j) cm = fmaxf(cm, v[j]);
    if (cm > m) {
      s *= expf(m - cm);  // first chunk: s = 0 and exp(-inf) = 0
      m = cm;
    }
#pragma unroll
    for (int j = 0; j < VEC; ++j) s += expf(v[j] - m);
  }
  // combine the threads: common maximum, sums rescaled to it
  const float wm = wave_max(m);
  s = wave_sum(m == -INFINITY ? 0.f : s * expf(m - wm));  // a thread past the row's end saw nothing
  const int w = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) { red_m[w] = wm; red_s[w] = s; }
  __syncthreads();  // also orders the read of z[label] above before the writes below
  const float M = fmaxf(fmaxf(red_m[0], red_m[1]), fmaxf(red_m[2], red_m[3]));
  float S = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) S += red_m[i] == -INFINITY ? 0.f : red_s[i] * expf(red_m[i] - M);
  const float lse = M + logf(S);
  if (threadIdx.x == 0) row_loss[row] = valid ? (lse - z_label) * scale : 0.f;
  const float sc = valid ? scale : 0.f;
  for (int c = threadIdx.x * VEC; c < S_voc; c += ROW_THREADS * VEC) {
    float v[VEC];
    load_vec<T, VEC>(zr + c, v);
#pragma unroll
    for (int j = 0; j < VEC; ++j) v[j] = (expf(v[j] - lse) - (c + j == label ? 1.f : 0.f)) * sc;
    store_vec<T, VEC>(zr + c, v);
  }
}

// out[0] = sum of n values, fixed order: strided partial sums per thread, then a tree.
__global__ __launch_bounds__(ROW_THREADS) void sum_rows_kernel(const float* __restrict__ v, float* __restrict__ out, int n) {
  __shared__ float red[ROW_THREADS];
  float s = 0.f;
  for (int i = threadIdx.x; i < n; i += ROW_THREADS) s += v[i];
  red[threadIdx.x] = s;
  __syncthreads();
  for (int o = ROW_THREADS / 2; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) out[0] = red[0];
}

inline bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

#define BF_LAUNCH_CHECK()                                                                  \
  do {                                                                                     \
    hipError_t e_ = hipGetLastError();                                                     \
    if (e_ != hipSuccess) { set_error("kernel launch failed: %s", hipGetErrorString(e_)); return BF_EDEVICE; } \
  } while (0)

}  // namespace

bf_status embedding_fwd(int dtype, int n_rows, int S_seq, int S_voc, int h, const int32_t* tok, const float* e_tok,
                        const float* e_pos, void* x, hipStream_t st) {
  if (n_rows < 1 || S_seq < 1 || S_voc < 1 || h < 1 || !tok || !e_tok || !e_pos || !x) { set_error("embedding_fwd: bad argument"); return BF_EINVAL; }
  const bool vec = h % 4 == 0 && aligned16(e_tok) && aligned16(e_pos) && aligned16(x);
  if (dtype == BF_BF16) {
    if (vec) embedding_fwd_kernel<bf16_t, 4><<<n_rows, ROW_THREADS, 0, st>>>(tok, e_tok, e_pos, (bf16_t*)x, S_seq, S_voc, h);
    else embedding_fwd_kernel<bf16_t, 1><<<n_rows, ROW_THREADS, 0, st>>>(tok, e_tok, e_pos, (bf16_t*)x, S_seq, S_voc, h);
  } else {
    if (vec) embedding_fwd_kernel<float, 4><<<n_rows, ROW_THREADS, 0, st>>>(tok, e_tok, e_pos, (float*)x, S_seq, S_voc, h);
    else embedding_fwd_kernel<float, 1><<<n_rows, ROW_THREADS, 0, st>>>(tok, e_tok, e_pos, (float*)x, S_seq, S_voc, h);
  }
  BF_LAUNCH_CHECK();
  return BF_OK;
}

bf_status embedding_bwd(int dtype, int S_mb, int S_seq, int S_voc, int h, const int32_t* tok, const void* d, float* g_tok,
                        float* g_pos, int accumulate_pos, hipStream_t st) {
  if (S_mb < 1 || S_seq < 1 || S_voc < 1 || h < 1 || !tok || !d || !g_tok || !g_pos) { set_error("embedding_bwd: bad argument"); return BF_EINVAL; }
  const int n_rows = S_mb * S_seq;
  const bool vec = h % 4 == 0 && aligned16(d) && aligned16(g_tok) && aligned16(g_pos);
  if (dtype == BF_BF16) {
    if (vec) {
      embedding_bwd_tok_kernel<bf16_t, 4><<<n_rows, ROW_THREADS, 0, st>>>(tok, (const bf16_t*)d, g_tok, n_rows, S_voc, h);
      embedding_bwd_pos_kernel<bf16_t, 4><<<S_seq, ROW_THREADS, 0, st>>>((const bf16_t*)d, g_pos, S_mb, S_seq, h, accumulate_pos);
    } else {
      embedding_bwd_tok_kernel<bf16_t, 1><<<n_rows, ROW_THREADS, 0, st>>>(tok, (const bf16_t*)d, g_tok, n_rows, S_voc, h);
      embedding_bwd_pos_kernel<bf16_t, 1><<<S_seq, ROW_THREADS, 0, st>>>((const bf16_t*)d, g_pos, S_mb, S_seq, h, accumulate_pos);
    }
  } else {
    if (vec) {
      embedding_bwd_tok_kernel<float, 4><<<n_rows, ROW_THREADS, 0, st>>>(tok, (const float*)d, g_tok, n_rows, S_voc, h);
      embedding_bwd_pos_kernel<float, 4><<<S_seq, ROW_THREADS, 0, st>>>((const float*)d, g_pos, S_mb, S_seq, h, accumulate_pos);
    } else {
      embedding_bwd_tok_kernel<float, 1><<<n_rows, ROW_THREADS, 0, st>>>(tok, (const float*)d, g_tok, n_rows, S_voc, h);
      embedding_bwd_pos_kernel<float, 1><<<S_seq, ROW_THREADS, 0, st>>>((const float*)d, g_pos, S_mb, S_seq, h, accumulate_pos);
    }
  }
  BF_LAUNCH_CHECK();
  return BF_OK;
}

bf_status ce_loss(int dtype, int n_rows, int S_voc, void* z, const int32_t* labels, float scale, float* row_loss,
                  float* loss_out, hipStream_t st) {
  if (n_rows < 1 || S_voc < 1 || !z || !labels || !row_loss || !loss_out) { set_error("ce_loss: bad argument"); return BF_EINVAL; }
  const bool vec = S_voc % 4 == 0 && aligned16(z);
  if (dtype == BF_BF16) {
    if (vec) ce_loss_kernel<bf16_t, 4><<<n_rows, ROW_THREADS, 0, st>>>((bf16_t*)z, labels, row_loss, S_voc, scale);
    else ce_loss_kernel<bf16_t, 1><<<n_rows, ROW_THREADS, 0, st>>>((bf16_t*)z, labels, row_loss, S_voc, scale);
  } else {
    if (vec) ce_loss_kernel<float, 4><<<n_rows, ROW_THREADS, 0, st>>>((float*)z, labels, row_loss, S_voc, scale);
    else ce_loss_kernel<float, 1><<<n_rows, ROW_THREADS, 0, st>>>((float*)z, labels, row_loss, S_voc, scale);
  }
  BF_LAUNCH_CHECK();
  sum_rows_kernel<<<1, ROW_THREADS, 0, st>>>(row_loss, loss_out, n_rows);
  BF_LAUNCH_CHECK();
  return BF_OK;
}

}  // namespace bf
