// Plain FMA GEMM for the fp32 parity configuration (and as an any-shape fallback).
// 64x64 output tile per workgroup, 16-deep K slices through LDS, 4x4 outputs per thread,
// fp32 accumulation in ascending k: deterministic.  Not a performance path.
#include "kernels.h"
#include "gelu.h"

namespace swarm {
namespace {

constexpr int TM = 64, TN = 64, TK = 16;

template <typename T>
__global__ __launch_bounds__(256) void gemm_generic_kernel(GemmArgs g) {
  __shared__ float As[TK][TM + 1];
  __shared__ float Bs[TK][TN + 1];
  const T* A = (const T*)g.A;
  const T* B = (const T*)g.B;
  const int m0 = blockIdx.y * TM, n0 = blockIdx.x * TN;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

  for (int k0 = 0; k0 < g.K; k0 += TK) {
    for (int e = threadIdx.x; e < TM * TK; e += 256) {
      int mm, kk;
      if (g.a_trans) { mm = e % TM; kk = e / TM; } else { kk = e % TK; mm = e / TK; }
      const int m = m0 + mm, k = k0 + kk;
      float v = 0.f;
      if (m < g.M && k < g.K)
        v = Elem<T>::load(g.a_trans ? A + (size_t)k * g.lda + m : A + (size_t)m * g.lda + k);
      As[kk][mm] = v;
    }
    for (int e = threadIdx.x; e < TN * TK; e += 256) {
      int nn, kk;
      if (g.b_trans) { nn = e % TN; kk = e / TN; } else { kk = e % TK; nn = e / TK; }
      const int n = n0 + nn, k = k0 + kk;
      float v = 0.f;
      if (n < g.N && k < g.K)
        v = Elem<T>::load(g.b_trans ? B + (size_t)k * g.ldb + n : B + (size_t)n * g.ldb + k);
      Bs[kk][nn] = v;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < TK; ++kk) {
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
    const int m = m0 + ty * 4 + i;
    if (m >= g.M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n >= g.N) continue;
      float v = acc[i][j];
      switch (g.epilogue) {
        case EPI_STORE:
          Elem<T>::store((T*)g.C + (size_t)m * g.ldc + n, v);
          break;
        case EPI_BIAS:
          Elem<T>::store((T*)g.C + (size_t)m * g.ldc + n, v + Elem<T>::load((const T*)g.bias + n));
          break;
        case EPI_BIAS_RESID:
          Elem<T>::store((T*)g.C + (size_t)m * g.ldc + n,
                         v + Elem<T>::load((const T*)g.bias + n) +
                             Elem<T>::load((const T*)g.aux + (size_t)m * g.ldaux + n));
          break;
        case EPI_BIAS_GELU: {
          const float u = v + Elem<T>::load((const T*)g.bias + n);
          if (g.C2) Elem<T>::store((T*)g.C2 + (size_t)m * g.ldc2 + n, u);
          Elem<T>::store((T*)g.C + (size_t)m * g.ldc + n, gelu_f(u));
          break;
        }
        case EPI_DGELU:
          Elem<T>::store((T*)g.C + (size_t)m * g.ldc + n,
                         v * gelu_grad_f(Elem<T>::load((const T*)g.aux + (size_t)m * g.ldaux + n)));
          break;
        case EPI_ACCUM_F32:
          ((float*)g.C)[(size_t)m * g.ldc + n] += v;
          break;
      }
    }
  }
}

}  // namespace

swarm_status gemm_generic(const GemmArgs& g, bool bf16, hipStream_t st) {
  dim3 grid((g.N + TN - 1) / TN, (g.M + TM - 1) / TM);
  if (bf16)
    hipLaunchKernelGGL(gemm_generic_kernel<bf16_raw>, grid, dim3(256), 0, st, g);
  else
    hipLaunchKernelGGL(gemm_generic_kernel<float>, grid, dim3(256), 0, st, g);
  return launch_status();
}

swarm_status gemm_f32(const GemmArgs& g, hipStream_t st) { return gemm_generic(g, false, st); }

}  // namespace swarm
