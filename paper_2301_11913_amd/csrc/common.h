// Shared device/host helpers for the gfx950 pipeline-stage kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "swarm_stage.h"

namespace swarm {

typedef __bf16 bf16;
typedef uint16_t bf16_raw;

constexpr int kWave = 64;   // CDNA4 wavefront width

__device__ __forceinline__ float bf16_bits_to_float(uint32_t bits16) {
  return __uint_as_float(bits16 << 16);
}

// fp32 -> bf16 bit pattern, round-to-nearest-even (finite inputs).
__device__ __forceinline__ uint32_t float_to_bf16_bits(float x) {
  uint32_t u = __float_as_uint(x);
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return float_to_bf16_bits(lo) | (float_to_bf16_bits(hi) << 16);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
  static __device__ __forceinline__ float load(const float* p) { return *p; }
  static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct Elem<bf16_raw> {
  static __device__ __forceinline__ float load(const bf16_raw* p) { return bf16_bits_to_float(*p); }
  static __device__ __forceinline__ void store(bf16_raw* p, float v) { *p = (bf16_raw)float_to_bf16_bits(v); }
};

// Butterfly reductions over the 64 lanes of a wavefront.
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v = fmaxf(v, __shfl_xor(v, m, 64));
  return v;
}

// x / s, correctly rounded, for many x and one s (the block scale of the boundary codec, whose codes are
// rint(x / s) and have to come out bit for bit).  The correctly rounded fp32 division is the sequence
//   r0 = rcp(s); r = fma(fma(-s, r0, 1), r0, r0); q = x r; q = fma(fma(-s, q, x), r, q); q = fma(fma(-s, q, x), r, q)
// wrapped in operand scaling and a fix-up that only act when an exponent is extreme.  With s in [2^-100, 2^100]
// they act only on numerators below 2^-103 or quotients in the subnormal range: there |x / s| < 1/8, and whatever
// the unscaled sequence returns for it also rounds to the code 0.  So r is computed once per block and every
// element costs one multiplication and four fused multiply-adds; any other s takes the plain division.
struct BlockDivisor {
  float s, r;
  bool plain;
  __device__ __forceinline__ explicit BlockDivisor(float scale) : s(scale) {
    const uint32_t biased = (__float_as_uint(scale) >> 23) & 0xFFu;
    plain = biased - 27u > 200u;
    const float r0 = __builtin_amdgcn_rcpf(scale);
    r = __builtin_fmaf(__builtin_fmaf(-scale, r0, 1.0f), r0, r0);
  }
  // a value whose rintf() equals rintf(x / s)
  __device__ __forceinline__ float quotient(float x) const {
    if (plain) return x / s;
    float q = x * r;
    q = __builtin_fmaf(__builtin_fmaf(-s, q, x), r, q);
    return __builtin_fmaf(__builtin_fmaf(-s, q, x), r, q);
  }
};

// Block scale of the boundary codec as stored: fp32, or (s16) its bf16 rounding as a 16-bit pattern.  The codes
// always divide by the value that is stored, so the encoder rounds the scale BEFORE it quantises.
__device__ __forceinline__ float block_scale_rounded(float s, bool s16) {
  return s16 ? __uint_as_float(float_to_bf16_bits(s) << 16) : s;
}
__device__ __forceinline__ void block_scale_store(void* scales, size_t i, float s, bool s16) {
  if (s16) reinterpret_cast<uint16_t*>(scales)[i] = (uint16_t)(__float_as_uint(s) >> 16);
  else reinterpret_cast<float*>(scales)[i] = s;
}
__device__ __forceinline__ float block_scale_load(const void* scales, size_t i, bool s16) {
  return s16 ? __uint_as_float((uint32_t) reinterpret_cast<const uint16_t*>(scales)[i] << 16)
             : reinterpret_cast<const float*>(scales)[i];
}

inline swarm_status launch_status() {
  return hipGetLastError() == hipSuccess ? SWARM_OK : SWARM_ERR_LAUNCH;
}

// A kernel that wants more than 64 KB of dynamic LDS has to be told so once per device.  `done` is the caller's
// static record (one per kernel instantiation), indexed by device.
constexpr int kMaxDevices = 64;
struct LdsOptIn {
  bool done[kMaxDevices] = {};
};
inline swarm_status lds_opt_in(const void* kernel, size_t bytes, LdsOptIn& rec) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SWARM_ERR_LAUNCH;
  if (!rec.done[dev]) {
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess)
      return SWARM_ERR_LAUNCH;
    rec.done[dev] = true;
  }
  return SWARM_OK;
}

}  // namespace swarm
