// Accumulator epilogues shared by the GEMM kernels: bias, residual, GeLU forward
// (tanh form) and GeLU backward, fp32 main-grad accumulation.
#pragma once
#include "common.h"

namespace bf {

// tanh(x) = 1 - 2 / (1 + e^(2x)) on the hardware exp2 / reciprocal (about 1 ulp each).  The
// absolute error is ~1e-7, which is what matters here: tanh only enters as (1 + t) and (1 - t^2).
// Saturates correctly: e^(2x) -> inf gives 1, -> 0 gives -1.
__device__ __forceinline__ float tanh_fast(float x) {
  const float e = __builtin_amdgcn_exp2f(x * 2.8853900817779268f);  // 2 log2(e)
  return 1.0f - 2.0f * __builtin_amdgcn_rcpf(1.0f + e);
}

__device__ __forceinline__ float gelu_f(float u) {
  const float k0 = 0.7978845608028654f, k1 = 0.044715f;
  return 0.5f * u * (1.0f + tanh_fast(k0 * (u + k1 * u * u * u)));
}

__device__ __forceinline__ float gelu_grad_f(float u) {
  const float k0 = 0.7978845608028654f, k1 = 0.044715f;
  const float t = tanh_fast(k0 * (u + k1 * u * u * u));
  const float dt = (1.0f - t * t) * k0 * (1.0f + 3.0f * k1 * u * u);
  return 0.5f * (1.0f + t) + 0.5f * u * dt;
}

// Applies epilogue EPI to one accumulator value at (m, n) and stores it.
// TO is the activation type for E_NONE..E_GELU_BWD and float for E_ACCUM.
template <int EPI, typename TO>
__device__ __forceinline__ void epilogue_store(float acc, size_t m, size_t n, size_t ldc, TO* C, const float* bias,
                                               const TO* R, TO* C2, int accumulate) {
  const size_t idx = m * ldc + n;
  if (EPI == E_NONE) {
    C[idx] = (TO)acc;
  } else if (EPI == E_BIAS) {
    C[idx] = (TO)(acc + bias[n]);
  } else if (EPI == E_BIAS_RES) {
    C[idx] = (TO)(acc + bias[n] + (float)R[idx]);
  } else if (EPI == E_BIAS_GELU) {
    // the pre-activation is stored in TO first and the GeLU is taken of the stored
    // value, which is what the backward will read
    const TO u = (TO)(acc + bias[n]);
    C[idx] = u;
    C2[idx] = (TO)gelu_f((float)u);
  } else if (EPI == E_GELU_BWD) {
    C[idx] = (TO)(acc * gelu_grad_f((float)R[idx]));
  } else {  // E_ACCUM
    C[idx] = (TO)(accumulate ? (float)C[idx] + acc : acc);
  }
}

}  // namespace bf
