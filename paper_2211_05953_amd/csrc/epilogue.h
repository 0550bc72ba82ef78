// Accumulator epilogues shared by the GEMM kernels: bias, residual, GeLU forward
// (tanh form) and GeLU backward, fp32 main-grad accumulation.
#pragma once
#include "common.h"

namespace bf {

// GeLU in its tanh form, gelu(u) = u/2 (1 + tanh z) with z = sqrt(2/pi) (u + 0.044715 u^3), written
// through the logistic function: (1 + tanh z) / 2 = s := 1 / (1 + e^(-2z)), so that
//   gelu(u)  = u s
//   gelu'(u) = s + u s (1 - s) 2 z'(u),   2 z'(u) = 2 sqrt(2/pi) (1 + 3 * 0.044715 u^2)
// on the hardware exp2 / reciprocal (about 1 ulp each; s has an absolute error of ~1e-7).  Five
// (nine) plain operations and two transcendental ones per element: the epilogues of the two MLP
// products run them on 128 elements per lane with no MFMA work beside them.
// Saturates correctly: e^(-2z) -> inf gives s = 0, -> 0 gives s = 1.
__device__ __forceinline__ float gelu_logistic(float u, float u2) {
  const float c0 = -2.0f * 0.7978845608028654f * 1.4426950408889634f, c1 = c0 * 0.044715f;
  const float e = __builtin_amdgcn_exp2f(u * fmaf(u2, c1, c0));  // e^(-2z)
  return __builtin_amdgcn_rcpf(1.0f + e);
}

__device__ __forceinline__ float gelu_f(float u) { return u * gelu_logistic(u, u * u); }

__device__ __forceinline__ float gelu_grad_f(float u) {
  const float d0 = 2.0f * 0.7978845608028654f, d1 = d0 * 3.0f * 0.044715f;
  const float u2 = u * u;
  const float s = gelu_logistic(u, u2);
  const float w = u * fmaf(u2, d1, d0);  // u 2 z'(u)
  return fmaf(s, fmaf(-s, w, w), s);     // s (1 + w (1 - s))
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
