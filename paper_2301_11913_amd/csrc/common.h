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
