// Activations of the MLP scorer, shared by the bulk scoring kernels and the per-token scorer of
// the append step.
#pragma once

#include <hip/hip_runtime.h>

namespace lkv {

constexpr int kActSilu = 0;
constexpr int kActGelu = 1;

// Exact-form GELU, 0.5 z (1 + erf(z / sqrt 2)), branch free.  erf uses the five-term rational
// approximation 7.1.26 of Abramowitz & Stegun, erf(x) = 1 - (a1 t + ... + a5 t^5) exp(-x^2),
// t = 1 / (1 + p x) for x >= 0, absolute error below 1.5e-7 (plus fp32 rounding).  Written as
// max(z, 0) - |z|/2 * poly(t) * exp(-z^2/2), which has no cancellation for negative z.  The
// library erff costs several times more issue slots (and branches), which made the kernel
// VALU-bound instead of HBM-bound.
__device__ __forceinline__ float gelu_erf(float z) {
  const float az = fabsf(z);
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f * 0.70710678118654752f, az, 1.0f));
  // -poly(t) / 2: the factor of the last line is folded into the coefficients
  float p = fmaf(-0.5f * 1.061405429f, t, 0.5f * 1.453152027f);
  p = fmaf(p, t, -0.5f * 1.421413741f);
  p = fmaf(p, t, 0.5f * 0.284496736f);
  p = fmaf(p, t, -0.5f * 0.254829592f);
  p *= t;
  const float e = __builtin_amdgcn_exp2f((z * z) * (-0.5f * 1.4426950408889634f));   // exp(-z^2 / 2)
  return fmaf(az, p * e, fmaxf(z, 0.f));
}

template <int kAct>
__device__ __forceinline__ float activation(float z) {
  if (kAct == kActSilu) {
    // z * sigmoid(z); exp2 overflow for very negative z gives rcp(inf) = 0
    return z * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-1.4426950408889634f * z));
  } else {
    return gelu_erf(z);
  }
}

}  // namespace lkv
