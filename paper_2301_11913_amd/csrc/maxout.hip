// Maxout over non-overlapping windows of k consecutive features (appendix "Compression-Aware Architectures",
// paragraph "Maxout compression"), forward and backward.  Streaming, HBM-bound: a thread owns 8 consecutive
// input features (one 16-byte load for bf16) when k divides 8, else one window.
#include "kernels.h"

namespace swarm {
namespace {

template <typename T> __device__ __forceinline__ void ld8(const T* p, float (&x)[8]);
template <> __device__ __forceinline__ void ld8<bf16_raw>(const bf16_raw* p, float (&x)[8]) {
  const uint4 v = *reinterpret_cast<const uint4*>(p);
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    x[2 * i] = __uint_as_float(w[i] << 16);
    x[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
  }
}
template <> __device__ __forceinline__ void ld8<float>(const float* p, float (&x)[8]) {
  const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
  x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
}

// K in {2, 4, 8}: thread = 8 inputs -> 8/K outputs
template <typename T, int K>
__global__ __launch_bounds__(256) void maxout_fwd_vec_kernel(const T* __restrict__ a, T* __restrict__ z, size_t nchunk) {
  for (size_t c = (size_t)blockIdx.x * 256 + threadIdx.x; c < nchunk; c += (size_t)gridDim.x * 256) {
    float x[8];
    ld8<T>(a + c * 8, x);
#pragma unroll
    for (int w = 0; w < 8 / K; ++w) {
      float m = x[w * K];
#pragma unroll
      for (int i = 1; i < K; ++i) m = fmaxf(m, x[w * K + i]);
      Elem<T>::store(z + c * (8 / K) + w, m);
    }
  }
}

template <typename T, int K>
__global__ __launch_bounds__(256) void maxout_bwd_vec_kernel(const T* __restrict__ a, const T* __restrict__ dz,
                                                             T* __restrict__ da, size_t nchunk) {
  for (size_t c = (size_t)blockIdx.x * 256 + threadIdx.x; c < nchunk; c += (size_t)gridDim.x * 256) {
    float x[8];
    ld8<T>(a + c * 8, x);
#pragma unroll
    for (int w = 0; w < 8 / K; ++w) {
      int arg = 0;
      float m = x[w * K];
#pragma unroll
      for (int i = 1; i < K; ++i)
        if (x[w * K + i] > m) { m = x[w * K + i]; arg = i; }      // strict: ties keep the first
      const float g = Elem<T>::load(dz + c * (8 / K) + w);
#pragma unroll
      for (int i = 0; i < K; ++i) Elem<T>::store(da + c * 8 + w * K + i, i == arg ? g : 0.0f);
    }
  }
}

// any k: thread = one window
template <typename T>
__global__ __launch_bounds__(256) void maxout_fwd_any_kernel(const T* __restrict__ a, T* __restrict__ z, size_t nwin,
                                                             int k) {
  for (size_t w = (size_t)blockIdx.x * 256 + threadIdx.x; w < nwin; w += (size_t)gridDim.x * 256) {
    float m = Elem<T>::load(a + w * k);
    for (int i = 1; i < k; ++i) m = fmaxf(m, Elem<T>::load(a + w * k + i));
    Elem<T>::store(z + w, m);
  }
}

template <typename T>
__global__ __launch_bounds__(256) void maxout_bwd_any_kernel(const T* __restrict__ a, const T* __restrict__ dz,
                                                             T* __restrict__ da, size_t nwin, int k) {
  for (size_t w = (size_t)blockIdx.x * 256 + threadIdx.x; w < nwin; w += (size_t)gridDim.x * 256) {
    int arg = 0;
    float m = Elem<T>::load(a + w * k);
    for (int i = 1; i < k; ++i) {
      const float v = Elem<T>::load(a + w * k + i);
      if (v > m) { m = v; arg = i; }
    }
    const float g = Elem<T>::load(dz + w);
    for (int i = 0; i < k; ++i) Elem<T>::store(da + w * k + i, i == arg ? g : 0.0f);
  }
}

int grid_for(size_t n) { return (int)std::min<size_t>(std::max<size_t>((n + 255) / 256, 1), 256 * 16); }

template <typename T>
swarm_status fwd_t(const T* a, T* z, int rows, int n, int k, hipStream_t st) {
  const size_t nwin = (size_t)rows * n;
  const bool vec = ((uintptr_t)a & 15) == 0 && (nwin * k) % 8 == 0;
  if (vec && k == 2)
    hipLaunchKernelGGL((maxout_fwd_vec_kernel<T, 2>), dim3(grid_for(nwin * k / 8)), dim3(256), 0, st, a, z, nwin * k / 8);
  else if (vec && k == 4)
    hipLaunchKernelGGL((maxout_fwd_vec_kernel<T, 4>), dim3(grid_for(nwin * k / 8)), dim3(256), 0, st, a, z, nwin * k / 8);
  else if (vec && k == 8)
    hipLaunchKernelGGL((maxout_fwd_vec_kernel<T, 8>), dim3(grid_for(nwin * k / 8)), dim3(256), 0, st, a, z, nwin * k / 8);
  else
    hipLaunchKernelGGL(maxout_fwd_any_kernel<T>, dim3(grid_for(nwin)), dim3(256), 0, st, a, z, nwin, k);
  return launch_status();
}

template <typename T>
swarm_status bwd_t(const T* a, const T* dz, T* da, int rows, int n, int k, hipStream_t st) {
  const size_t nwin = (size_t)rows * n;
  const bool vec = ((uintptr_t)a & 15) == 0 && (nwin * k) % 8 == 0;
  if (vec && k == 2)
    hipLaunchKernelGGL((maxout_bwd_vec_kernel<T, 2>), dim3(grid_for(nwin * k / 8)), dim3(256), 0, st, a, dz, da, nwin * k / 8);
  else if (vec && k == 4)
    hipLaunchKernelGGL((maxout_bwd_vec_kernel<T, 4>), dim3(grid_for(nwin * k / 8)), dim3(256), 0, st, a, dz, da, nwin * k / 8);
  else if (vec && k == 8)
    hipLaunchKernelGGL((maxout_bwd_vec_kernel<T, 8>), dim3(grid_for(nwin * k / 8)), dim3(256), 0, st, a, dz, da, nwin * k / 8);
  else
    hipLaunchKernelGGL(maxout_bwd_any_kernel<T>, dim3(grid_for(nwin)), dim3(256), 0, st, a, dz, da, nwin, k);
  return launch_status();
}

}  // namespace

swarm_status maxout_fwd(const void* a, void* z, int T, int n, int k, bool bf16, hipStream_t st) {
  if (T < 1 || n < 1 || k < 1) return SWARM_ERR_SHAPE;
  return bf16 ? fwd_t<bf16_raw>((const bf16_raw*)a, (bf16_raw*)z, T, n, k, st)
              : fwd_t<float>((const float*)a, (float*)z, T, n, k, st);
}

swarm_status maxout_bwd(const void* a, const void* dz, void* da, int T, int n, int k, bool bf16, hipStream_t st) {
  if (T < 1 || n < 1 || k < 1) return SWARM_ERR_SHAPE;
  return bf16 ? bwd_t<bf16_raw>((const bf16_raw*)a, (const bf16_raw*)dz, (bf16_raw*)da, T, n, k, st)
              : bwd_t<float>((const float*)a, (const float*)dz, (float*)da, T, n, k, st);
}

}  // namespace swarm
