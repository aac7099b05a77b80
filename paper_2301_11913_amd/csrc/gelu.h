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
// |error| <= 1.5e-7, far below a bf16 ulp), written in terms of u = sqrt(2) x so that no instruction is spent on
// x itself; the exponential is shared with the normal density.  erf_abs = erf(|u| / sqrt 2), ex = exp(-u^2 / 2).
__device__ __forceinline__ void erf_and_exp(float u, float& erf_abs, float& ex) {
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f * 0.70710678118654752440f, fabsf(u), 1.0f));
  const float poly =
      fmaf(fmaf(fmaf(fmaf(1.061405429f, t, -1.453152027f), t, 1.421413741f), t, -0.284496736f), t, 0.254829592f) * t;
  ex = __builtin_amdgcn_exp2f((-0.5f * 1.4426950408889634f) * u * u);
  erf_abs = fmaf(-poly, ex, 1.0f);
}

__device__ __forceinline__ float gelu_fast(float u) {
  float e, ex;
  erf_and_exp(u, e, ex);
  const float h = 0.5f * u;
  return fmaf(fabsf(h), e, h);             // 0.5 u (1 + erf(u / sqrt 2)): the sign of erf is the sign of u
}

__device__ __forceinline__ float gelu_grad_fast(float u) {
  float e, ex;
  erf_and_exp(u, e, ex);
  const float cdf = fmaf(copysignf(0.5f, u), e, 0.5f);
  return fmaf(u * 0.39894228040143267794f, ex, cdf);
}

}  // namespace swarm
