// HBM-bound kernels of the layer: LayerNorm forward/backward, column sums for bias
// gradients, fused Adam with low-precision recast, initialisation helpers.
// Row kernels: one 256-thread workgroup per token row, 16-byte vector accesses when
// the row length allows, wavefront (64-lane) shuffles + one LDS hop for the reductions.
// Column kernels: fixed reduction order, so results do not depend on scheduling.
#include "common.h"

namespace bf {

namespace {

constexpr int ROW_THREADS = 256;

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// Sum over a 256-thread workgroup; every thread gets the result. `red` holds 4 floats.
__device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  const int w = threadIdx.x >> 6;
  __syncthreads();  // protects `red` against the previous use
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __syncthreads();
  return red[0] + red[1] + red[2] + red[3];
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

// ------------------------------------------------------------------ LayerNorm forward
template <typename T, int VEC>
__global__ __launch_bounds__(ROW_THREADS) void ln_fwd_kernel(const T* __restrict__ x, const float* __restrict__ g,
                                                             const float* __restrict__ b, T* __restrict__ y,
                                                             float* __restrict__ stats, int h, float eps) {
  __shared__ float red[4];
  const size_t row = blockIdx.x;
  const T* xr = x + row * (size_t)h;
  T* yr = y + row * (size_t)h;
  float s = 0.f;
  for (int i = threadIdx.x * VEC; i < h; i += ROW_THREADS * VEC) {
    float v[VEC];
    load_vec<T, VEC>(xr + i, v);
#pragma unroll
    for (int j = 0; j < VEC; ++j) s += v[j];
  }
  const float mean = block_sum(s, red) / (float)h;
  float q = 0.f;
  for (int i = threadIdx.x * VEC; i < h; i += ROW_THREADS * VEC) {
    float v[VEC];
    load_vec<T, VEC>(xr + i, v);
#pragma unroll
    for (int j = 0; j < VEC; ++j) {
      const float d = v[j] - mean;
      q += d * d;
    }
  }
  const float var = block_sum(q, red) / (float)h;
  const float rstd = 1.0f / sqrtf(var + eps);
  if (threadIdx.x == 0) {
    stats[2 * row] = mean;
    stats[2 * row + 1] = rstd;
  }
  for (int i = threadIdx.x * VEC; i < h; i += ROW_THREADS * VEC) {
    float v[VEC], gg[VEC], bb[VEC], o[VEC];
    load_vec<T, VEC>(xr + i, v);
    load_vec<float, VEC>(g + i, gg);
    load_vec<float, VEC>(b + i, bb);
#pragma unroll
    for (int j = 0; j < VEC; ++j) o[j] = (v[j] - mean) * rstd * gg[j] + bb[j];
    store_vec<T, VEC>(yr + i, o);
  }
}

// Rows of at most ROW_THREADS * VEC * NIT elements stay in registers: the row is read once and the
// three passes (mean, variance, output) run on the copy.
template <typename T, int VEC, int NIT>
__global__ __launch_bounds__(ROW_THREADS) void ln_fwd_reg_kernel(const T* __restrict__ x, const float* __restrict__ g,
                                                                 const float* __restrict__ b, T* __restrict__ y,
                                                                 float* __restrict__ stats, int h, float eps) {
  __shared__ float red[4];
  const size_t row = blockIdx.x;
  const T* xr = x + row * (size_t)h;
  T* yr = y + row * (size_t)h;
  float v[NIT][VEC];
  float s = 0.f;
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    const int i = (it * ROW_THREADS + (int)threadIdx.x) * VEC;
    if (i < h) {
      load_vec<T, VEC>(xr + i, v[it]);
#pragma unroll
      for (int j = 0; j < VEC; ++j) s += v[it][j];
    }
  }
  const float mean = block_sum(s, red) / (float)h;
  float q = 0.f;
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    const int i = (it * ROW_THREADS + (int)threadIdx.x) * VEC;
    if (i < h) {
#pragma unroll
      for (int j = 0; j < VEC; ++j) {
        const float d = v[it][j] - mean;
        q += d * d;
      }
    }
  }
  const float var = block_sum(q, red) / (float)h;
  const float rstd = 1.0f / sqrtf(var + eps);
  if (threadIdx.x == 0) {
    stats[2 * row] = mean;
    stats[2 * row + 1] = rstd;
  }
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    const int i = (it * ROW_THREADS + (int)threadIdx.x) * VEC;
    if (i < h) {
      float gg[VEC], bb[VEC], o[VEC];
      load_vec<float, VEC>(g + i, gg);
      load_vec<float, VEC>(b + i, bb);
#pragma unroll
      for (int j = 0; j < VEC; ++j) o[j] = (v[it][j] - mean) * rstd * gg[j] + bb[j];
      store_vec<T, VEC>(yr + i, o);
    }
  }
}

// ------------------------------------------------------ LayerNorm backward, input gradient
// dx = rstd * (dxhat - mean(dxhat) - xhat * mean(dxhat * xhat)) [+ dres],  dxhat = dy * g
template <typename T, int VEC>
__global__ __launch_bounds__(ROW_THREADS) void ln_bwd_dx_kernel(const T* __restrict__ dy, const T* __restrict__ x,
                                                                const float* __restrict__ g,
                                                                const float* __restrict__ stats,
                                                                const T* __restrict__ dres, T* __restrict__ dx, int h) {
  __shared__ float red[4];
  const size_t row = blockIdx.x;
  const T* dyr = dy + row * (size_t)h;
  const T* xr = x + row * (size_t)h;
  const float mean = stats[2 * row], rstd = stats[2 * row + 1];
  float s1 = 0.f, s2 = 0.f;
  for (int i = threadIdx.x * VEC; i < h; i += ROW_THREADS * VEC) {
    float d[VEC], v[VEC], gg[VEC];
    load_vec<T, VEC>(dyr + i, d);
    load_vec<T, VEC>(xr + i, v);
    load_vec<float, VEC>(g + i, gg);
#pragma unroll
    for (int j = 0; j < VEC; ++j) {
      const float dxh = d[j] * gg[j];
      s1 += dxh;
      s2 += dxh * ((v[j] - mean) * rstd);
    }
  }
  s1 = block_sum(s1, red) / (float)h;
  s2 = block_sum(s2, red) / (float)h;
  for (int i = threadIdx.x * VEC; i < h; i += ROW_THREADS * VEC) {
    float d[VEC], v[VEC], gg[VEC], r[VEC], o[VEC];
    load_vec<T, VEC>(dyr + i, d);
    load_vec<T, VEC>(xr + i, v);
    load_vec<float, VEC>(g + i, gg);
    if (dres) {
      load_vec<T, VEC>(dres + row * (size_t)h + i, r);
    } else {
#pragma unroll
      for (int j = 0; j < VEC; ++j) r[j] = 0.f;
    }
#pragma unroll
    for (int j = 0; j < VEC; ++j) {
      const float xh = (v[j] - mean) * rstd;
      o[j] = rstd * (d[j] * gg[j] - s1 - xh * s2) + r[j];
    }
    store_vec<T, VEC>(dx + row * (size_t)h + i, o);
  }
}

// The same with dy and x of the row held in registers between the two passes.
template <typename T, int VEC, int NIT>
__global__ __launch_bounds__(ROW_THREADS) void ln_bwd_dx_reg_kernel(const T* __restrict__ dy, const T* __restrict__ x,
                                                                    const float* __restrict__ g,
                                                                    const float* __restrict__ stats,
                                                                    const T* __restrict__ dres, T* __restrict__ dx, int h) {
  __shared__ float red[4];
  const size_t row = blockIdx.x;
  const T* dyr = dy + row * (size_t)h;
  const T* xr = x + row * (size_t)h;
  const float mean = stats[2 * row], rstd = stats[2 * row + 1];
  float dh[NIT][VEC], xh[NIT][VEC];  // dy * g and the normalised input
  float s1 = 0.f, s2 = 0.f;
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    const int i = (it * ROW_THREADS + (int)threadIdx.x) * VEC;
    if (i < h) {
      float gg[VEC];
      load_vec<T, VEC>(dyr + i, dh[it]);
      load_vec<T, VEC>(xr + i, xh[it]);
      load_vec<float, VEC>(g + i, gg);
#pragma unroll
      for (int j = 0; j < VEC; ++j) {
        dh[it][j] *= gg[j];
        xh[it][j] = (xh[it][j] - mean) * rstd;
        s1 += dh[it][j];
        s2 += dh[it][j] * xh[it][j];
      }
    }
  }
  s1 = block_sum(s1, red) / (float)h;
  s2 = block_sum(s2, red) / (float)h;
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    const int i = (it * ROW_THREADS + (int)threadIdx.x) * VEC;
    if (i < h) {
      float r[VEC], o[VEC];
      if (dres) {
        load_vec<T, VEC>(dres + row * (size_t)h + i, r);
      } else {
#pragma unroll
        for (int j = 0; j < VEC; ++j) r[j] = 0.f;
      }
#pragma unroll
      for (int j = 0; j < VEC; ++j) o[j] = rstd * (dh[it][j] - s1 - xh[it][j] * s2) + r[j];
      store_vec<T, VEC>(dx + row * (size_t)h + i, o);
    }
  }
}

// ------------------------------------------- LayerNorm backward, everything in one pass
// dx as above, and the three column reductions that go with a LayerNorm in the backward pass
// (dg = sum_t dy xhat, db = sum_t dy, and the column sums of the stored dx, which are the bias gradient
// of the linear layer that produced the LayerNorm's input) without reading dy and x a second time:
// a workgroup walks R consecutive rows, a thread keeps the three sums of its NIT * VEC columns in
// registers and the workgroup leaves one row of partial sums in `part` ([P][3][h], P = workgroups);
// ln_bwd_finish_kernel adds the P rows up in ascending order.  The next row's dy / x / dres are
// requested before the current row's reductions, so the row-to-row chain does not expose HBM latency.
// Sum over the workgroup of two values at once; `red` holds 8 floats.
__device__ __forceinline__ void block_sum2(float& a, float& b, float* red) {
  a = wave_sum(a);
  b = wave_sum(b);
  const int w = threadIdx.x >> 6;
  __syncthreads();  // protects `red` against the previous use
  if ((threadIdx.x & 63) == 0) { red[w] = a; red[4 + w] = b; }
  __syncthreads();
  a = red[0] + red[1] + red[2] + red[3];
  b = red[4] + red[5] + red[6] + red[7];
}

template <typename T, int VEC, int NIT>
__global__ __launch_bounds__(ROW_THREADS) void ln_bwd_fused_kernel(const T* __restrict__ dy, const T* __restrict__ x,
                                                                   const float* __restrict__ g, const float* __restrict__ stats,
                                                                   const T* __restrict__ dres, T* __restrict__ dx,
                                                                   float* __restrict__ part, int T_rows, int h, int R) {
  __shared__ float red[8];
  typedef Vec<T, VEC> V;
  const int r0 = blockIdx.x * R, r1 = min(r0 + R, T_rows);
  float gg[NIT][VEC], ag[NIT][VEC], ab[NIT][VEC], ac[NIT][VEC];
  int col[NIT];
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    col[it] = (it * ROW_THREADS + (int)threadIdx.x) * VEC;
    if (col[it] < h) load_vec<float, VEC>(g + col[it], gg[it]);
#pragma unroll
    for (int j = 0; j < VEC; ++j) ag[it][j] = ab[it][j] = ac[it][j] = 0.f;
  }
  V ndy[NIT], nx[NIT], nres[NIT];  // the next row, as it comes from memory
  auto fetch = [&](int row) {
#pragma unroll
    for (int it = 0; it < NIT; ++it)
      if (col[it] < h) {
        ndy[it] = *reinterpret_cast<const V*>(dy + (size_t)row * h + col[it]);
        nx[it] = *reinterpret_cast<const V*>(x + (size_t)row * h + col[it]);
        if (dres) nres[it] = *reinterpret_cast<const V*>(dres + (size_t)row * h + col[it]);
      }
  };
  if (r0 < r1) fetch(r0);
  for (int row = r0; row < r1; ++row) {
    const float mean = stats[2 * row], rstd = stats[2 * row + 1];
    float d[NIT][VEC], xh[NIT][VEC], rr[NIT][VEC];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int it = 0; it < NIT; ++it)
      if (col[it] < h) {
#pragma unroll
        for (int j = 0; j < VEC; ++j) {
          d[it][j] = (float)ndy[it].v[j];
          xh[it][j] = ((float)nx[it].v[j] - mean) * rstd;
          rr[it][j] = dres ? (float)nres[it].v[j] : 0.f;
          const float dh = d[it][j] * gg[it][j];
          s1 += dh;
          s2 += dh * xh[it][j];
        }
      }
    if (row + 1 < r1) fetch(row + 1);
    block_sum2(s1, s2, red);
    s1 /= (float)h;
    s2 /= (float)h;
#pragma unroll
    for (int it = 0; it < NIT; ++it)
      if (col[it] < h) {
        V o;
#pragma unroll
        for (int j = 0; j < VEC; ++j) {
          o.v[j] = (T)(rstd * (d[it][j] * gg[it][j] - s1 - xh[it][j] * s2) + rr[it][j]);
          ag[it][j] += d[it][j] * xh[it][j];
          ab[it][j] += d[it][j];
          ac[it][j] += (float)o.v[j];
        }
        *reinterpret_cast<V*>(dx + (size_t)row * h + col[it]) = o;
      }
  }
  float* p = part + (size_t)blockIdx.x * 3 * h;
#pragma unroll
  for (int it = 0; it < NIT; ++it)
    if (col[it] < h) {
      store_vec<float, VEC>(p + col[it], ag[it]);
      store_vec<float, VEC>(p + h + col[it], ab[it]);
      store_vec<float, VEC>(p + 2 * (size_t)h + col[it], ac[it]);
    }
}

// out_q[c] = (accumulate ? out_q[c] : 0) + sum_{b < P} part[b][q][c] for q = 0 (dg), 1 (db), 2 (dcs, may be null),
// rows added in ascending order: 16 threads x 4 columns (256 contiguous bytes of a partial row) by 16 row
// groups per workgroup, the groups meet in LDS in order.  h is a multiple of 4, so a thread's four columns
// belong to one output.
__global__ __launch_bounds__(256) void ln_bwd_finish_kernel(const float* __restrict__ part, int P, int h, float* __restrict__ dg,
                                                            float* __restrict__ db, float* __restrict__ dcs, int accumulate) {
  __shared__ float red[16][16][4];
  const int cx = threadIdx.x & 15, ry = threadIdx.x >> 4;
  const int c3 = (blockIdx.x * 16 + cx) * 4;  // first of the thread's columns of the [3 h] row of partial sums
  const int per = (P + 15) / 16, b0 = ry * per, b1 = min(b0 + per, P);
  float t[4] = {0.f, 0.f, 0.f, 0.f};
  if (c3 < 3 * h) {
#pragma unroll 4
    for (int b = b0; b < b1; ++b) {
      float u[4];
      load_vec<float, 4>(part + (size_t)b * 3 * h + c3, u);
#pragma unroll
      for (int j = 0; j < 4; ++j) t[j] += u[j];
    }
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) red[ry][cx][j] = t[j];
  __syncthreads();
  if (ry == 0 && c3 < 3 * h) {
    const int q = c3 / h, c = c3 - q * h;
    float* out = q == 0 ? dg : q == 1 ? db : dcs;
    if (out) {
      float v[4] = {0.f, 0.f, 0.f, 0.f};
      if (accumulate) load_vec<float, 4>(out + c, v);
#pragma unroll
      for (int r = 0; r < 16; ++r)
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] += red[r][cx][j];
      store_vec<float, 4>(out + c, v);
    }
  }
}

// Compute units of the current device (256 on MI355X).
inline int compute_units() {
  static const int n = [] {
    int dev = 0, cu = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cu < 1) cu = 256;
    return cu;
  }();
  return n;
}

// ---------------------------------------------------- column reductions (fixed order)
// Workgroup = CG column groups x RG row groups (CG * RG = 256); thread (cx, ry) owns VEC adjacent
// columns and rows ry, ry + RG, ...  Partial sums meet in LDS and are added in ascending ry.
// A workgroup covers CG * VEC columns: narrow enough that the few thousand columns of a bias
// or LayerNorm gradient still spread over all compute units, wide enough (>= 128 bytes per
// row) to keep the row reads in whole cache lines.  When that gives fewer workgroups than compute
// units the launcher halves the width (CG = 4: two workgroups share each 128-byte line) and sets
// `pair`: workgroups go to the 8 XCDs round-robin, so the two halves of a line are given to
// workgroups b and b + 8, which share an XCD and its L2.
// MODE 0: out[c] = sum_t dY[t,c]
// MODE 1: dg[c] = sum_t dY[t,c] * xhat[t,c],  db[c] = sum_t dY[t,c]
template <typename T, int VEC, int MODE, int CG>
__global__ __launch_bounds__(256) void col_reduce_kernel(const T* __restrict__ dY, const T* __restrict__ x,
                                                         const float* __restrict__ stats, float* __restrict__ out0,
                                                         float* __restrict__ out1, int T_rows, int N, int accumulate,
                                                         int pair) {
  constexpr int RG = 256 / CG;
  __shared__ float part[MODE == 1 ? 2 : 1][RG][CG * VEC + 1];
  const int cx = threadIdx.x % CG, ry = threadIdx.x / CG;
  const int b = blockIdx.x;
  const int blk = pair ? (b & 7) * 2 + ((b >> 3) & 1) + (b >> 4) * 16 : b;  // a bijection on every 16 workgroups
  const int c0 = (blk * CG + cx) * VEC;
  float a0[VEC], a1[VEC];
#pragma unroll
  for (int j = 0; j < VEC; ++j) a0[j] = a1[j] = 0.f;
  if (c0 < N) {
    // UN rows in flight per thread: the loads of a batch are issued together, the sums keep their order
    constexpr int UN = 8;
    int t = ry;
    for (; t + (UN - 1) * RG < T_rows; t += UN * RG) {
      float d[UN][VEC], v[UN][VEC], mean[UN], rstd[UN];
#pragma unroll
      for (int u = 0; u < UN; ++u) {
        load_vec<T, VEC>(dY + (size_t)(t + u * RG) * N + c0, d[u]);
        if (MODE == 1) {
          load_vec<T, VEC>(x + (size_t)(t + u * RG) * N + c0, v[u]);
          mean[u] = stats[2 * (t + u * RG)];
          rstd[u] = stats[2 * (t + u * RG) + 1];
        }
      }
#pragma unroll
      for (int u = 0; u < UN; ++u)
#pragma unroll
        for (int j = 0; j < VEC; ++j) {
          if (MODE == 1) {
            a0[j] += d[u][j] * ((v[u][j] - mean[u]) * rstd[u]);
            a1[j] += d[u][j];
          } else {
            a0[j] += d[u][j];
          }
        }
    }
    for (; t < T_rows; t += RG) {
      float d[VEC];
      load_vec<T, VEC>(dY + (size_t)t * N + c0, d);
      if (MODE == 1) {
        float v[VEC];
        load_vec<T, VEC>(x + (size_t)t * N + c0, v);
        const float mean = stats[2 * t], rstd = stats[2 * t + 1];
#pragma unroll
        for (int j = 0; j < VEC; ++j) {
          a0[j] += d[j] * ((v[j] - mean) * rstd);
          a1[j] += d[j];
        }
      } else {
#pragma unroll
        for (int j = 0; j < VEC; ++j) a0[j] += d[j];
      }
    }
  }
#pragma unroll
  for (int j = 0; j < VEC; ++j) {
    part[0][ry][cx * VEC + j] = a0[j];
    if (MODE == 1) part[MODE == 1 ? 1 : 0][ry][cx * VEC + j] = a1[j];
  }
  __syncthreads();
  for (int c = threadIdx.x; c < CG * VEC; c += 256) {
    const int col = blk * CG * VEC + c;
    if (col >= N) continue;
    float s0 = 0.f, s1 = 0.f;
#pragma unroll 8
    for (int r = 0; r < RG; ++r) {
      s0 += part[0][r][c];
      if (MODE == 1) s1 += part[MODE == 1 ? 1 : 0][r][c];
    }
    out0[col] = accumulate ? out0[col] + s0 : s0;
    if (MODE == 1) out1[col] = accumulate ? out1[col] + s1 : s1;
  }
}

template <typename T, int VEC, int MODE>
void launch_col_reduce(const void* dY, const void* x, const float* stats, float* out0, float* out1, int T_rows, int N,
                       int accumulate, hipStream_t st) {
  constexpr int CG = 8;  // 8 x VEC columns per workgroup, 32 row groups
  const int blocks = (N + CG * VEC - 1) / (CG * VEC);
  if (VEC >= 4 && blocks < compute_units()) {
    const int nb = (N + 4 * VEC - 1) / (4 * VEC);
    col_reduce_kernel<T, VEC, MODE, 4><<<nb, 256, 0, st>>>((const T*)dY, (const T*)x, stats, out0, out1, T_rows, N, accumulate, nb % 16 == 0);
    return;
  }
  col_reduce_kernel<T, VEC, MODE, CG><<<blocks, 256, 0, st>>>((const T*)dY, (const T*)x, stats, out0, out1, T_rows, N, accumulate, 0);
}

// ------------------------------------------------------------------------- fused Adam
// One pass: m, v, w updated in fp32; bf16 copy of w rewritten (mixed precision, App. A.1).
// The bias corrections c1 = 1 / (1 - beta1^t), c2 = 1 / (1 - beta2^t) come from the host, or, when
// t_dev is given, are taken in double from the step count stored on the device: a launch recorded
// in a HIP graph then follows the counter from replay to replay.
template <int VEC>
__global__ __launch_bounds__(256) void adam_kernel(size_t n, float* __restrict__ w, float* __restrict__ m,
                                                   float* __restrict__ v, const float* __restrict__ g,
                                                   bf16_t* __restrict__ w_lp, float lr, float beta1, float beta2,
                                                   float eps, float wd, float c1, float c2, float omb1, float omb2,
                                                   const int* __restrict__ t_dev) {
  if (t_dev) {
    const double t = (double)*t_dev;
    c1 = (float)(1.0 / (1.0 - pow((double)beta1, t)));
    c2 = (float)(1.0 / (1.0 - pow((double)beta2, t)));
  }
  const size_t stride = (size_t)gridDim.x * blockDim.x * VEC;
  for (size_t i = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * VEC; i < n; i += stride) {
    float ww[VEC], mm[VEC], vv[VEC], gg[VEC];
    load_vec<float, VEC>(w + i, ww);
    load_vec<float, VEC>(m + i, mm);
    load_vec<float, VEC>(v + i, vv);
    load_vec<float, VEC>(g + i, gg);
#pragma unroll
    for (int j = 0; j < VEC; ++j) {
      mm[j] = beta1 * mm[j] + omb1 * gg[j];
      vv[j] = beta2 * vv[j] + omb2 * gg[j] * gg[j];
      const float mhat = mm[j] * c1, vhat = vv[j] * c2;
      ww[j] = ww[j] - lr * (mhat / (sqrtf(vhat) + eps) + wd * ww[j]);
    }
    store_vec<float, VEC>(w + i, ww);
    store_vec<float, VEC>(m + i, mm);
    store_vec<float, VEC>(v + i, vv);
    if (w_lp) store_vec<bf16_t, VEC>(w_lp + i, ww);
  }
}

template <int VEC>
__global__ __launch_bounds__(256) void cast_kernel(size_t n, const float* __restrict__ src, bf16_t* __restrict__ dst) {
  const size_t stride = (size_t)gridDim.x * blockDim.x * VEC;
  for (size_t i = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * VEC; i < n; i += stride) {
    float t[VEC];
    load_vec<float, VEC>(src + i, t);
    store_vec<bf16_t, VEC>(dst + i, t);
  }
}

__global__ __launch_bounds__(256) void fill_kernel(size_t n, float* __restrict__ dst, float value) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = value;
}

__device__ __forceinline__ uint64_t mix64(uint64_t z) {
  z += 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

// Counter-based N(0, std): two uniforms from a hash of (seed, index), Box-Muller.
__global__ __launch_bounds__(256) void init_normal_kernel(size_t n, float* __restrict__ dst, uint64_t seed, float std) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
    const uint64_t r = mix64(seed ^ mix64(i));
    const float u1 = ((float)(uint32_t)(r >> 40) + 1.0f) * (1.0f / 16777217.0f);  // (0, 1)
    const float u2 = (float)(uint32_t)((r >> 8) & 0xFFFFFF) * (1.0f / 16777216.0f);
    dst[i] = std * sqrtf(-2.0f * logf(u1)) * cosf(6.283185307179586f * u2);
  }
}

inline int grid_for(size_t n, int per_block) {
  size_t g = (n + per_block - 1) / per_block;
  if (g > 256 * 16) g = 256 * 16;  // 256 CUs, a few workgroups each; kernels grid-stride
  if (g < 1) g = 1;
  return (int)g;
}

inline bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

}  // namespace

#define BF_LAUNCH_CHECK()                                 \
  do {                                                    \
    hipError_t e_ = hipGetLastError();                    \
    if (e_ != hipSuccess) {                               \
      set_error("kernel launch failed: %s (%s:%d)", hipGetErrorString(e_), __FILE__, __LINE__); \
      return BF_EDEVICE;                                  \
    }                                                     \
  } while (0)

bf_status layernorm_fwd(int dtype, int T, int h, const void* x, const float* g, const float* b, float eps, void* y,
                        float* stats, hipStream_t st) {
  if (T < 1 || h < 1 || !x || !g || !b || !y || !stats) { set_error("layernorm_fwd: bad argument"); return BF_EINVAL; }
  if (dtype == BF_BF16) {
    const bool vec = h % 8 == 0 && aligned16(x) && aligned16(y) && aligned16(g) && aligned16(b);
    if (vec && h <= ROW_THREADS * 8) ln_fwd_reg_kernel<bf16_t, 8, 1><<<T, ROW_THREADS, 0, st>>>((const bf16_t*)x, g, b, (bf16_t*)y, stats, h, eps);
    else if (vec && h <= ROW_THREADS * 16) ln_fwd_reg_kernel<bf16_t, 8, 2><<<T, ROW_THREADS, 0, st>>>((const bf16_t*)x, g, b, (bf16_t*)y, stats, h, eps);
    else if (vec && h <= ROW_THREADS * 32) ln_fwd_reg_kernel<bf16_t, 8, 4><<<T, ROW_THREADS, 0, st>>>((const bf16_t*)x, g, b, (bf16_t*)y, stats, h, eps);
    else if (vec) ln_fwd_kernel<bf16_t, 8><<<T, ROW_THREADS, 0, st>>>((const bf16_t*)x, g, b, (bf16_t*)y, stats, h, eps);
    else ln_fwd_kernel<bf16_t, 1><<<T, ROW_THREADS, 0, st>>>((const bf16_t*)x, g, b, (bf16_t*)y, stats, h, eps);
  } else {
    const bool vec = h % 4 == 0 && aligned16(x) && aligned16(y) && aligned16(g) && aligned16(b);
    if (vec) ln_fwd_kernel<float, 4><<<T, ROW_THREADS, 0, st>>>((const float*)x, g, b, (float*)y, stats, h, eps);
    else ln_fwd_kernel<float, 1><<<T, ROW_THREADS, 0, st>>>((const float*)x, g, b, (float*)y, stats, h, eps);
  }
  BF_LAUNCH_CHECK();
  return BF_OK;
}

template <typename T, int VEC>
static void launch_ln_bwd(int T_rows, int h, const void* dy, const void* x, const float* g, const float* stats,
                          const void* dres, void* dx, float* dg, float* db, int accumulate, hipStream_t st) {
  if (VEC > 1 && h <= ROW_THREADS * VEC)
    ln_bwd_dx_reg_kernel<T, VEC, 1><<<T_rows, ROW_THREADS, 0, st>>>((const T*)dy, (const T*)x, g, stats, (const T*)dres, (T*)dx, h);
  else if (VEC > 1 && h <= ROW_THREADS * VEC * 2)
    ln_bwd_dx_reg_kernel<T, VEC, 2><<<T_rows, ROW_THREADS, 0, st>>>((const T*)dy, (const T*)x, g, stats, (const T*)dres, (T*)dx, h);
  else if (VEC > 1 && h <= ROW_THREADS * VEC * 4)
    ln_bwd_dx_reg_kernel<T, VEC, 4><<<T_rows, ROW_THREADS, 0, st>>>((const T*)dy, (const T*)x, g, stats, (const T*)dres, (T*)dx, h);
  else
    ln_bwd_dx_kernel<T, VEC><<<T_rows, ROW_THREADS, 0, st>>>((const T*)dy, (const T*)x, g, stats, (const T*)dres, (T*)dx, h);
  launch_col_reduce<T, VEC, 1>(dy, x, stats, dg, db, T_rows, h, accumulate, st);
}

// Workgroups of the one-pass LayerNorm backward (each walks a run of consecutive rows).  One per compute unit is
// the measured optimum at 2048 rows of 8192: 128 and 192 take 35 % and 11 % longer although they write fewer
// partial sums.
constexpr int LN_BWD_WGS = 256;
size_t layernorm_bwd_part_elems(int T, int h) {
  const int R = (T + LN_BWD_WGS - 1) / LN_BWD_WGS, P = (T + R - 1) / R;
  return (size_t)P * 3 * (size_t)h;
}

template <typename T, int VEC>
static bool launch_ln_bwd_fused(int T_rows, int h, const void* dy, const void* x, const float* g, const float* stats,
                                const void* dres, void* dx, float* dg, float* db, float* dcs, float* part, int accumulate,
                                hipStream_t st) {
  const int nit = (h + ROW_THREADS * VEC - 1) / (ROW_THREADS * VEC);
  if (nit > 4) return false;
  // at most 256 workgroups (one per compute unit), each a run of consecutive rows
  const int R = (T_rows + LN_BWD_WGS - 1) / LN_BWD_WGS, P = (T_rows + R - 1) / R;
#define BF_LN_FUSED(N) ln_bwd_fused_kernel<T, VEC, N><<<P, ROW_THREADS, 0, st>>>((const T*)dy, (const T*)x, g, stats, (const T*)dres, (T*)dx, part, T_rows, h, R)
  switch (nit) {
    case 1: BF_LN_FUSED(1); break;
    case 2: BF_LN_FUSED(2); break;
    case 3: BF_LN_FUSED(3); break;
    default: BF_LN_FUSED(4); break;
  }
#undef BF_LN_FUSED
  ln_bwd_finish_kernel<<<(3 * h + 63) / 64, 256, 0, st>>>(part, P, h, dg, db, dcs, accumulate);
  return true;
}

bf_status layernorm_bwd(int dtype, int T, int h, const void* dy, const void* x, const float* g, const float* stats,
                        const void* dres, void* dx, float* dg, float* db, int accumulate, hipStream_t st, float* dcs,
                        float* part) {
  if (T < 1 || h < 1 || !dy || !x || !g || !stats || !dx || !dg || !db) { set_error("layernorm_bwd: bad argument"); return BF_EINVAL; }
  const bool al = aligned16(dy) && aligned16(x) && aligned16(g) && aligned16(dx) && (!dres || aligned16(dres));
  if (part && al && aligned16(part) && aligned16(dg) && aligned16(db) && (!dcs || aligned16(dcs))) {
    // one pass over dy / x with the column reductions on the way (rows of up to 4 x 256 vectors)
    bool done = false;
    if (dtype == BF_BF16 && h % 8 == 0) done = launch_ln_bwd_fused<bf16_t, 8>(T, h, dy, x, g, stats, dres, dx, dg, db, dcs, part, accumulate, st);
    else if (dtype == BF_FP32 && h % 4 == 0) done = launch_ln_bwd_fused<float, 4>(T, h, dy, x, g, stats, dres, dx, dg, db, dcs, part, accumulate, st);
    if (done) {
      BF_LAUNCH_CHECK();
      return BF_OK;
    }
  }
  if (dcs) {
    // no scratch or an odd shape: the input gradient first, then its column sums as a pass of their own
    bf_status r = layernorm_bwd(dtype, T, h, dy, x, g, stats, dres, dx, dg, db, accumulate, st, nullptr, nullptr);
    if (r != BF_OK) return r;
    return colsum(dtype, T, h, dx, dcs, accumulate, st);
  }
  if (dtype == BF_BF16) {
    if (al && h % 8 == 0) launch_ln_bwd<bf16_t, 8>(T, h, dy, x, g, stats, dres, dx, dg, db, accumulate, st);
    else launch_ln_bwd<bf16_t, 1>(T, h, dy, x, g, stats, dres, dx, dg, db, accumulate, st);
  } else {
    if (al && h % 4 == 0) launch_ln_bwd<float, 4>(T, h, dy, x, g, stats, dres, dx, dg, db, accumulate, st);
    else launch_ln_bwd<float, 1>(T, h, dy, x, g, stats, dres, dx, dg, db, accumulate, st);
  }
  BF_LAUNCH_CHECK();
  return BF_OK;
}

bf_status colsum(int dtype, int T, int N, const void* dY, float* out, int accumulate, hipStream_t st) {
  if (T < 1 || N < 1 || !dY || !out) { set_error("colsum: bad argument"); return BF_EINVAL; }
  if (dtype == BF_BF16) {
    if (aligned16(dY) && N % 8 == 0) launch_col_reduce<bf16_t, 8, 0>(dY, nullptr, nullptr, out, nullptr, T, N, accumulate, st);
    else launch_col_reduce<bf16_t, 1, 0>(dY, nullptr, nullptr, out, nullptr, T, N, accumulate, st);
  } else {
    if (aligned16(dY) && N % 4 == 0) launch_col_reduce<float, 4, 0>(dY, nullptr, nullptr, out, nullptr, T, N, accumulate, st);
    else launch_col_reduce<float, 1, 0>(dY, nullptr, nullptr, out, nullptr, T, N, accumulate, st);
  }
  BF_LAUNCH_CHECK();
  return BF_OK;
}

__global__ __launch_bounds__(256) void colsum_finish_kernel(const float* __restrict__ part, int rows, int N, float* __restrict__ out,
                                                            int accumulate) {
  const int n = blockIdx.x * 256 + threadIdx.x;
  if (n >= N) return;
  float t = accumulate ? out[n] : 0.f;
  for (int r = 0; r < rows; ++r) t += part[(size_t)r * N + n];
  out[n] = t;
}

bf_status colsum_finish(const float* part, int rows, int N, float* out, int accumulate, hipStream_t st) {
  if (!part || !out || rows < 1 || N < 1) { set_error("colsum_finish: bad argument"); return BF_EINVAL; }
  colsum_finish_kernel<<<(N + 255) / 256, 256, 0, st>>>(part, rows, N, out, accumulate);
  BF_LAUNCH_CHECK();
  return BF_OK;
}

__global__ __launch_bounds__(256) void attn_bias_finish_kernel(const float* __restrict__ pq, int rows_q, const float* __restrict__ pkv,
                                                               int rows_kv, int h, float* __restrict__ out, int accumulate) {
  const int n = blockIdx.x * 256 + threadIdx.x;
  if (n >= 3 * h) return;
  float t = accumulate ? out[n] : 0.f;
  if (n < h)
    for (int r = 0; r < rows_q; ++r) t += pq[(size_t)r * h + n];
  else
    for (int r = 0; r < rows_kv; ++r) t += pkv[(size_t)r * 2 * h + (n - h)];
  out[n] = t;
}

bf_status attn_bias_finish(const float* pq, int rows_q, const float* pkv, int rows_kv, int h, float* out, int accumulate,
                           hipStream_t st) {
  if (!pq || !pkv || !out || rows_q < 1 || rows_kv < 1 || h < 1) { set_error("attn_bias_finish: bad argument"); return BF_EINVAL; }
  attn_bias_finish_kernel<<<(3 * h + 255) / 256, 256, 0, st>>>(pq, rows_q, pkv, rows_kv, h, out, accumulate);
  BF_LAUNCH_CHECK();
  return BF_OK;
}

// C = epilogue(sum of the planes of a split contraction), 8 adjacent columns per thread; planes added in ascending order
template <int EPI>
__global__ __launch_bounds__(256) void splitk_finish_kernel(int slices, size_t MN, int N, const float* __restrict__ part,
                                                            const float* __restrict__ bias, const bf16_t* __restrict__ R,
                                                            bf16_t* __restrict__ C) {
  const size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 8;
  if (i >= MN) return;
  float v[8];
  load_vec<float, 8>(part + i, v);
  for (int s = 1; s < slices; ++s) {
    float u[8];
    load_vec<float, 8>(part + (size_t)s * MN + i, u);
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] += u[j];
  }
  if (EPI == E_BIAS || EPI == E_BIAS_RES) {
    float b[8];
    load_vec<float, 8>(bias + (i % (size_t)N), b);
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] += b[j];
  }
  if (EPI == E_BIAS_RES) {
    float r[8];
    load_vec<bf16_t, 8>(R + i, r);
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] += r[j];
  }
  store_vec<bf16_t, 8>(C + i, v);
}

bf_status gemm_splitk_finish(int epi, int M, int N, int slices, const float* part, const float* bias, const void* R, void* C,
                             hipStream_t st) {
  if (M < 1 || N < 8 || N % 8 || slices < 2 || !part || !C) { set_error("gemm_splitk_finish: bad argument"); return BF_EINVAL; }
  if ((epi == E_BIAS || epi == E_BIAS_RES) && !bias) { set_error("gemm_splitk_finish: bias is null"); return BF_EINVAL; }
  if (epi == E_BIAS_RES && !R) { set_error("gemm_splitk_finish: residual is null"); return BF_EINVAL; }
  if (!aligned16(part) || !aligned16(C) || (bias && !aligned16(bias)) || (R && !aligned16(R))) {
    set_error("gemm_splitk_finish: operands must be 16-byte aligned");
    return BF_EINVAL;
  }
  const size_t MN = (size_t)M * N;
  const unsigned grid = (unsigned)((MN / 8 + 255) / 256);
  switch (epi) {
    case E_NONE: splitk_finish_kernel<E_NONE><<<grid, 256, 0, st>>>(slices, MN, N, part, bias, (const bf16_t*)R, (bf16_t*)C); break;
    case E_BIAS: splitk_finish_kernel<E_BIAS><<<grid, 256, 0, st>>>(slices, MN, N, part, bias, (const bf16_t*)R, (bf16_t*)C); break;
    case E_BIAS_RES: splitk_finish_kernel<E_BIAS_RES><<<grid, 256, 0, st>>>(slices, MN, N, part, bias, (const bf16_t*)R, (bf16_t*)C); break;
    default: set_error("gemm_splitk_finish: epilogue %d is not finished here", epi); return BF_EINVAL;
  }
  BF_LAUNCH_CHECK();
  return BF_OK;
}

__global__ void bump_step_kernel(int* t) { *t += 1; }

bf_status bump_step(int* t_dev, hipStream_t st) {
  bump_step_kernel<<<1, 1, 0, st>>>(t_dev);
  BF_LAUNCH_CHECK();
  return BF_OK;
}

bf_status adam_step(size_t n, float* w, float* m, float* v, const float* g, bf16_t* w_lp, int t, const int* t_dev, float lr,
                    float beta1, float beta2, float eps, float wd, hipStream_t st) {
  if (n == 0) return BF_OK;
  if (!w || !m || !v || !g || (!t_dev && t < 1)) { set_error("adam_step: bad argument"); return BF_EINVAL; }
  // bias corrections in double, applied as multipliers: here for a step count given by value, in the
  // kernel for one kept on the device
  const float c1 = t_dev ? 0.f : (float)(1.0 / (1.0 - pow((double)beta1, (double)t)));
  const float c2 = t_dev ? 0.f : (float)(1.0 / (1.0 - pow((double)beta2, (double)t)));
  const float omb1 = (float)(1.0 - (double)beta1), omb2 = (float)(1.0 - (double)beta2);
  const bool vec = n % 4 == 0 && aligned16(w) && aligned16(m) && aligned16(v) && aligned16(g) &&
                   (!w_lp || ((uintptr_t)w_lp & 7) == 0);
  // One workgroup of four waves per compute unit streams fastest (measured on 1.6e9 parameters: 5.2 TB/s
  // against 4.8 with 16 workgroups per unit, 5.0 with two, 3.5 with half a workgroup's threads).
  const int grid4 = grid_for(n, 1024) < compute_units() ? grid_for(n, 1024) : compute_units();
  if (vec) adam_kernel<4><<<grid4, 256, 0, st>>>(n, w, m, v, g, w_lp, lr, beta1, beta2, eps, wd, c1, c2, omb1, omb2, t_dev);
  else adam_kernel<1><<<grid_for(n, 256), 256, 0, st>>>(n, w, m, v, g, w_lp, lr, beta1, beta2, eps, wd, c1, c2, omb1, omb2, t_dev);
  BF_LAUNCH_CHECK();
  return BF_OK;
}

bf_status cast_f32_to_bf16(size_t n, const float* src, bf16_t* dst, hipStream_t st) {
  if (n == 0) return BF_OK;
  const bool vec = n % 4 == 0 && aligned16(src) && ((uintptr_t)dst & 7) == 0;
  if (vec) cast_kernel<4><<<grid_for(n, 1024), 256, 0, st>>>(n, src, dst);
  else cast_kernel<1><<<grid_for(n, 256), 256, 0, st>>>(n, src, dst);
  BF_LAUNCH_CHECK();
  return BF_OK;
}

bf_status fill_f32(size_t n, float* dst, float value, hipStream_t st) {
  if (n == 0) return BF_OK;
  fill_kernel<<<grid_for(n, 256), 256, 0, st>>>(n, dst, value);
  BF_LAUNCH_CHECK();
  return BF_OK;
}

namespace {
struct AddSegs { int n; size_t off[8]; size_t cnt[8]; };

// dst += src over up to eight element ranges of each of gridDim.y equally laid out layers
__global__ __launch_bounds__(256) void add_segments_kernel(size_t layer_stride, AddSegs sg, float* __restrict__ dst,
                                                           const float* __restrict__ src) {
  const size_t base = (size_t)blockIdx.y * layer_stride;
  for (int k = 0; k < sg.n; ++k) {
    float* d = dst + base + sg.off[k];
    const float* a = src + base + sg.off[k];
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < sg.cnt[k]; i += (size_t)gridDim.x * 256) d[i] += a[i];
  }
}
}  // namespace

bf_status add_segments(int n_layers, size_t layer_stride, int n_seg, const size_t* off, const size_t* cnt, float* dst,
                       const float* src, hipStream_t st) {
  if (n_layers < 1 || n_seg < 1 || n_seg > 8 || !dst || !src) { set_error("add_segments: bad arguments"); return BF_EINVAL; }
  AddSegs sg{};
  sg.n = n_seg;
  for (int k = 0; k < n_seg; ++k) { sg.off[k] = off[k]; sg.cnt[k] = cnt[k]; }
  add_segments_kernel<<<dim3(16, n_layers), 256, 0, st>>>(layer_stride, sg, dst, src);
  BF_LAUNCH_CHECK();
  return BF_OK;
}

bf_status init_normal(size_t n, float* dst, uint64_t seed, float std, hipStream_t st) {
  if (n == 0) return BF_OK;
  init_normal_kernel<<<grid_for(n, 256), 256, 0, st>>>(n, dst, seed, std);
  BF_LAUNCH_CHECK();
  return BF_OK;
}

}  // namespace bf
