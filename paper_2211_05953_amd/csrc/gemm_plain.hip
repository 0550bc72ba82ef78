// Plain GEMM: LDS-tiled fp32 FMA, any shape, any of the three operand layouts, both
// storage types.  It is the fp32-mode GEMM and the fallback for shapes the MFMA kernel
// does not take; it is not meant to be fast.
#include "common.h"
#include "epilogue.h"

namespace bf {

namespace {

constexpr int PT = 64;   // tile edge
constexpr int PK = 16;   // k step

// element (m, k) of op(A) is A[m * sam + k * sak]; (k, n) of op(B) is B[k * sbk + n * sbn]
template <typename TI, typename TO, int EPI>
__global__ __launch_bounds__(256) void gemm_plain_kernel(int M, int N, int K, const TI* __restrict__ A, size_t sam,
                                                         size_t sak, const TI* __restrict__ B, size_t sbk, size_t sbn,
                                                         TO* __restrict__ C, const float* __restrict__ bias,
                                                         const TO* __restrict__ R, TO* __restrict__ C2, int accumulate) {
  __shared__ float As[PK][PT + 1];
  __shared__ float Bs[PK][PT + 1];
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int m0 = blockIdx.y * PT, n0 = blockIdx.x * PT;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

  for (int k0 = 0; k0 < K; k0 += PK) {
    for (int e = threadIdx.x; e < PT * PK; e += 256) {
      // A tile: walk k fastest when A is k-contiguous, m fastest otherwise
      int mm, kk;
      if (sak == 1) { kk = e % PK; mm = e / PK; } else { mm = e % PT; kk = e / PT; }
      const int gm = m0 + mm, gk = k0 + kk;
      As[kk][mm] = (gm < M && gk < K) ? (float)A[(size_t)gm * sam + (size_t)gk * sak] : 0.f;
      int nn, kb;
      if (sbk == 1) { kb = e % PK; nn = e / PK; } else { nn = e % PT; kb = e / PT; }
      const int gn = n0 + nn, gkb = k0 + kb;
      Bs[kb][nn] = (gn < N && gkb < K) ? (float)B[(size_t)gkb * sbk + (size_t)gn * sbn] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < PK; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int gm = m0 + ty * 4 + i;
    if (gm >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int gn = n0 + tx * 4 + j;
      if (gn < N) epilogue_store<EPI, TO>(acc[i][j], gm, gn, N, C, bias, R, C2, accumulate);
    }
  }
}

template <typename TI, typename TO, int EPI>
void launch(int layout, const GemmArgs& a, hipStream_t st) {
  size_t sam, sak, sbk, sbn;
  if (layout == L_TN) { sam = 1; sak = a.M; } else { sam = a.K; sak = 1; }
  if (layout == L_NT) { sbk = 1; sbn = a.K; } else { sbk = a.N; sbn = 1; }
  dim3 grid((a.N + PT - 1) / PT, (a.M + PT - 1) / PT);
  gemm_plain_kernel<TI, TO, EPI><<<grid, 256, 0, st>>>(a.M, a.N, a.K, (const TI*)a.A, sam, sak, (const TI*)a.B, sbk, sbn,
                                                        (TO*)a.C, a.bias, (const TO*)a.R, (TO*)a.C2, a.accumulate);
}

template <typename T>
bf_status dispatch(int layout, int epi, const GemmArgs& a, hipStream_t st) {
  switch (epi) {
    case E_NONE: launch<T, T, E_NONE>(layout, a, st); break;
    case E_BIAS: launch<T, T, E_BIAS>(layout, a, st); break;
    case E_BIAS_RES: launch<T, T, E_BIAS_RES>(layout, a, st); break;
    case E_BIAS_GELU: launch<T, T, E_BIAS_GELU>(layout, a, st); break;
    case E_GELU_BWD: launch<T, T, E_GELU_BWD>(layout, a, st); break;
    case E_ACCUM: launch<T, float, E_ACCUM>(layout, a, st); break;
    default: set_error("gemm: unknown epilogue %d", epi); return BF_EINVAL;
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_error("gemm_plain launch failed: %s", hipGetErrorString(e)); return BF_EDEVICE; }
  return BF_OK;
}

}  // namespace

bf_status gemm_check(int layout, int epi, const GemmArgs& a) {
  if (a.M < 1 || a.N < 1 || a.K < 1 || !a.A || !a.B || !a.C) { set_error("gemm: bad size or null operand"); return BF_EINVAL; }
  if (layout < L_NN || layout > L_TN) { set_error("gemm: unknown layout %d", layout); return BF_EINVAL; }
  if ((epi == E_BIAS || epi == E_BIAS_RES || epi == E_BIAS_GELU) && !a.bias) { set_error("gemm: epilogue needs bias"); return BF_EINVAL; }
  if ((epi == E_BIAS_RES || epi == E_GELU_BWD) && !a.R) { set_error("gemm: epilogue needs R"); return BF_EINVAL; }
  if (epi == E_BIAS_GELU && !a.C2) { set_error("gemm: epilogue needs C2"); return BF_EINVAL; }
  return BF_OK;
}

bf_status gemm_plain(int dtype, int layout, int epi, const GemmArgs& a, hipStream_t st) {
  bf_status s = gemm_check(layout, epi, a);
  if (s != BF_OK) return s;
  if (a.n_seg > 1) {
    if (layout != L_TN) { set_error("gemm: segments go with the weight-gradient layout"); return BF_EINVAL; }
    const size_t es = dtype == BF_BF16 ? 2 : 4;
    for (int i = 0; i < a.n_seg; ++i) {
      GemmArgs b = a;
      b.n_seg = 1;
      b.A = (const char*)a.A + (size_t)i * a.seg_stride_a * es;
      b.B = (const char*)a.B + (size_t)i * a.seg_stride_b * es;
      b.accumulate = i > 0 ? 1 : a.accumulate;
      if ((s = gemm_plain(dtype, layout, epi, b, st)) != BF_OK) return s;
    }
    return BF_OK;
  }
  if (dtype == BF_BF16) return dispatch<bf16_t>(layout, epi, a, st);
  if (dtype == BF_FP32) return dispatch<float>(layout, epi, a, st);
  set_error("gemm: unknown dtype %d", dtype);
  return BF_EINVAL;
}

bf_status gemm(int dtype, int kernels, int layout, int epi, const GemmArgs& a, hipStream_t st) {
  if (a.colsum && layout != L_TN && epi != E_GELU_BWD) {
    set_error("gemm: column sums go with the weight-gradient layout or the GeLU-backward epilogue");
    return BF_EINVAL;
  }
  const uintptr_t al = (uintptr_t)a.A | (uintptr_t)a.B | (uintptr_t)a.C | (uintptr_t)a.R | (uintptr_t)a.C2 | (uintptr_t)a.bias;
  bf_status s;
  const bool seg_ok = a.n_seg <= 1 || ((a.seg_stride_a | a.seg_stride_b) & 7) == 0;  // 16-byte aligned segments
  if (dtype == BF_BF16 && kernels == BF_KERNELS_AUTO && (al & 15) == 0 && seg_ok && gemm_mfma_supported(layout, epi, a.M, a.N, a.K)) {
    s = gemm_check(layout, epi, a);
    if (s != BF_OK) return s;
    if (layout != L_TN && a.colsum && a.colsum_part) {
      // the epilogue leaves one row of partial column sums per row of tiles; add them up
      int rows = 0;
      GemmArgs b = a;
      b.colsum_rows = &rows;
      s = gemm_mfma(layout, epi, b, st);
      if (s != BF_OK) return s;
      return colsum_finish(a.colsum_part, rows, a.N, a.colsum, a.accumulate, st);
    }
    GemmArgs b = a;
    b.colsum_part = nullptr;
    const int slices = a.splitk_ws ? gemm_splitk_slices(layout, epi, a.M, a.N, a.K) : 1;
    if (slices > 1 && a.splitk_ws_elems >= (size_t)slices * a.M * a.N && ((uintptr_t)a.splitk_ws & 15) == 0) {
      // few tiles, long contraction: slices of K on more workgroups into fp32 planes, then the planes added in order
      b.C = a.splitk_ws;
      b.bias = nullptr;
      b.R = nullptr;
      b.C2 = nullptr;
      b.accumulate = 0;
      b.k_slices = slices;
      s = gemm_mfma(layout, E_ACCUM, b, st);
      if (s != BF_OK) return s;
      return gemm_splitk_finish(epi, a.M, a.N, slices, a.splitk_ws, a.bias, a.R, a.C, st);
    }
    s = gemm_mfma(layout, epi, b, st);
  } else {
    s = gemm_plain(dtype, layout, epi, a, st);
  }
  if (s != BF_OK || !a.colsum) return s;
  if (layout != L_TN) return colsum(dtype, a.M, a.N, a.C, a.colsum, a.accumulate, st);  // second pass over the stored output
  // The bias gradient beside the weight gradient: one pass of the column-reduction kernel per
  // segment.  (Taking the sums inside the MFMA product, as ones^T B on a few workgroups, was
  // measured: those workgroups run 10 % longer and end up as the stragglers of their rounds, which
  // costs the product 2 % and gains the step 0.1 %.)
  const size_t es = dtype == BF_BF16 ? 2 : 4;
  for (int i = 0; i < (a.n_seg > 1 ? a.n_seg : 1); ++i) {
    s = colsum(dtype, a.K, a.N, (const char*)a.B + (size_t)i * a.seg_stride_b * es, a.colsum, i > 0 ? 1 : a.accumulate, st);
    if (s != BF_OK) return s;
  }
  return BF_OK;
}

}  // namespace bf
