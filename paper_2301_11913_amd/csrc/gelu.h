// Exact (erf) GeLU and its derivative in fp32.
#pragma once
#include <hip/hip_runtime.h>

namespace swarm {

__device__ __forceinline__ float gelu_f(float u) {
  return 0.5f * u * (1.0f + erff(u * 0.70710678118654752440f));
}

// d/du [u Phi(u)] = Phi(u) + u phi(u)
__device__ __forceinline__ float gelu_grad_f(float u) {
  const float cdf = 0.5f * (1.0f + erff(u * 0.70710678118654752440f));
  const float pdf = 0.39894228040143267794f * __expf(-0.5f * u * u);
  return cdf + u * pdf;
}

// Cheaper variants for the bf16 GEMM epilogues: erf by the classical rational approximation
// erf(x) = 1 - (a1 t + ... + a5 t^5) exp(-x^2), t = 1/(1 + p x)  (Abramowitz & Stegun 7.1.26,
// |error| <= 1.5e-7, far below a bf16 ulp); the exponential is shared with the normal density.
__device__ __forceinline__ void erf_and_exp(float x, float& erf_x, float& exp_mx2) {
  const float ax = fabsf(x);
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, ax, 1.0f));
  const float poly =
      fmaf(fmaf(fmaf(fmaf(1.061405429f, t, -1.453152027f), t, 1.421413741f), t, -0.284496736f), t, 0.254829592f) * t;
  exp_mx2 = __builtin_amdgcn_exp2f(-1.4426950408889634f * ax * ax);
  erf_x = copysignf(1.0f - poly * exp_mx2, x);
}

__device__ __forceinline__ float gelu_fast(float u) {
  float e, ex;
  erf_and_exp(u * 0.70710678118654752440f, e, ex);
  return 0.5f * u * (1.0f + e);
}

__device__ __forceinline__ float gelu_grad_fast(float u) {
  float e, ex;   // ex = exp(-u^2/2)
  erf_and_exp(u * 0.70710678118654752440f, e, ex);
  return 0.5f * (1.0f + e) + u * 0.39894228040143267794f * ex;
}

}  // namespace swarm
