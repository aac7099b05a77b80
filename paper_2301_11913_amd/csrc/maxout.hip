// Maxout over non-overlapping windows of k consecutive features (appendix "Compression-Aware Architectures",
// paragraph "Maxout compression"), forward and backward, for the window sizes that are not fused into the LayerNorm
// kernels round them (2, 4 and 8 are: a window then lies inside one lane's 8 values).  A thread owns one window.
#include "kernels.h"

namespace swarm {
namespace {

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
  hipLaunchKernelGGL(maxout_fwd_any_kernel<T>, dim3(grid_for(nwin)), dim3(256), 0, st, a, z, nwin, k);
  return launch_status();
}

template <typename T>
swarm_status bwd_t(const T* a, const T* dz, T* da, int rows, int n, int k, hipStream_t st) {
  const size_t nwin = (size_t)rows * n;
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
