// Rotary position embedding and GeGLU as stand-alone streaming kernels (the two changes the appendix
// "Additional Details for Section 4.3" makes to the standard Transformer layer).  The bf16 stage fuses
// both into GEMM epilogues where it can; these kernels serve the fp32 path, shapes the fused GEMM does
// not take, and the backward rotation.
//
// Rotary: inside every head, the pair (x[2i], x[2i+1]) of q and of k at sequence position pos is rotated by
// the angle pos * 10000^(-2i/d_head).  GeGLU: u = [gate | up] (2f columns), g = gelu(gate) * up.
#include "gelu.h"
#include "kernels.h"

namespace swarm {

namespace {

template <typename T> struct Act;
template <> struct Act<float> {
  static __device__ __forceinline__ float gelu(float u) { return gelu_f(u); }
  static __device__ __forceinline__ float gelu_grad(float u) { return gelu_grad_f(u); }
};
template <> struct Act<bf16_raw> {
  static __device__ __forceinline__ float gelu(float u) { return gelu_fast(u); }
  static __device__ __forceinline__ float gelu_grad(float u) { return gelu_grad_fast(u); }
};

template <typename T> __device__ __forceinline__ void load8(const T* p, float (&x)[8]);
template <> __device__ __forceinline__ void load8<bf16_raw>(const bf16_raw* p, float (&x)[8]) {
  const uint4 v = *reinterpret_cast<const uint4*>(p);
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    x[2 * i] = __uint_as_float(w[i] << 16);
    x[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
  }
}
template <> __device__ __forceinline__ void load8<float>(const float* p, float (&x)[8]) {
  const float4 a = *reinterpret_cast<const float4*>(p);
  const float4 b = *reinterpret_cast<const float4*>(p + 4);
  x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
}
template <typename T> __device__ __forceinline__ void store8(T* p, const float (&x)[8]);
template <> __device__ __forceinline__ void store8<bf16_raw>(bf16_raw* p, const float (&x)[8]) {
  uint4 v;
  v.x = pack_bf16x2(x[0], x[1]); v.y = pack_bf16x2(x[2], x[3]);
  v.z = pack_bf16x2(x[4], x[5]); v.w = pack_bf16x2(x[6], x[7]);
  *reinterpret_cast<uint4*>(p) = v;
}
template <> __device__ __forceinline__ void store8<float>(float* p, const float (&x)[8]) {
  *reinterpret_cast<float4*>(p) = make_float4(x[0], x[1], x[2], x[3]);
  *reinterpret_cast<float4*>(p + 4) = make_float4(x[4], x[5], x[6], x[7]);
}

// table[pos][i] = (cos, sin) of pos * 10000^(-2i/dh), i < dh/2; angles in fp64, rounded once to fp32.
__global__ __launch_bounds__(256) void rope_table_kernel(float2* __restrict__ table, int S, int half) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= S * half) return;
  const int pos = idx / half, i = idx - pos * half;
  const double inv = exp2(-(double)i / (double)half * 13.287712379549449);   // log2(10000)
  const double ang = (double)pos * inv;
  table[idx] = make_float2((float)cos(ang), (float)sin(ang));
}

// In place on columns [0, 2d) of the rows of qkv [T, 3d] (q then k).  One thread = 8 consecutive columns
// = 4 pairs; sign = +1 rotates by the angle, -1 by its negative (the transpose, used on dq and dk).
template <typename T>
__global__ __launch_bounds__(256) void rope_apply_kernel(T* __restrict__ qkv, const float2* __restrict__ table,
                                                         int rows, int S, int d, int dh, float sign) {
  const int cpr = (2 * d) >> 3;                        // chunks per row
  const size_t n = (size_t)rows * cpr;
  for (size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x; idx < n; idx += (size_t)gridDim.x * 256) {
    const int row = (int)(idx / cpr), c = (int)(idx - (size_t)row * cpr);
    const int col = c * 8;
    const int pos = row % S;
    const int pair0 = (col % dh) >> 1;
    T* p = qkv + (size_t)row * 3 * d + col;
    float x[8], y[8];
    load8<T>(p, x);
    const float4 t0 = *reinterpret_cast<const float4*>(table + (size_t)pos * (dh >> 1) + pair0);
    const float4 t1 = *reinterpret_cast<const float4*>(table + (size_t)pos * (dh >> 1) + pair0 + 2);
    const float cs[4] = {t0.x, t0.z, t1.x, t1.z};
    const float sn[4] = {t0.y * sign, t0.w * sign, t1.y * sign, t1.w * sign};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      y[2 * i] = x[2 * i] * cs[i] - x[2 * i + 1] * sn[i];
      y[2 * i + 1] = x[2 * i] * sn[i] + x[2 * i + 1] * cs[i];
    }
    store8<T>(p, y);
  }
}

// g[t, j] = gelu(u[t, j]) * u[t, f + j]
template <typename T>
__global__ __launch_bounds__(256) void geglu_fwd_kernel(const T* __restrict__ u, T* __restrict__ g, int rows, int f) {
  const int cpr = f >> 3;
  const size_t n = (size_t)rows * cpr;
  for (size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x; idx < n; idx += (size_t)gridDim.x * 256) {
    const size_t row = idx / cpr;
    const int col = (int)(idx - row * cpr) * 8;
    float a[8], b[8], o[8];
    load8<T>(u + row * 2 * f + col, a);
    load8<T>(u + row * 2 * f + f + col, b);
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = Act<T>::gelu(a[i]) * b[i];
    store8<T>(g + row * f + col, o);
  }
}

// du[t, j] = dg[t, j] * u[t, f + j] * gelu'(u[t, j]);  du[t, f + j] = dg[t, j] * gelu(u[t, j])
template <typename T>
__global__ __launch_bounds__(256) void geglu_bwd_kernel(const T* __restrict__ dg, const T* __restrict__ u,
                                                        T* __restrict__ du, int rows, int f) {
  const int cpr = f >> 3;
  const size_t n = (size_t)rows * cpr;
  for (size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x; idx < n; idx += (size_t)gridDim.x * 256) {
    const size_t row = idx / cpr;
    const int col = (int)(idx - row * cpr) * 8;
    float a[8], b[8], g[8], o1[8], o2[8];
    load8<T>(u + row * 2 * f + col, a);
    load8<T>(u + row * 2 * f + f + col, b);
    load8<T>(dg + row * f + col, g);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      o1[i] = g[i] * b[i] * Act<T>::gelu_grad(a[i]);
      o2[i] = g[i] * Act<T>::gelu(a[i]);
    }
    store8<T>(du + row * 2 * f + col, o1);
    store8<T>(du + row * 2 * f + f + col, o2);
  }
}

int stream_grid(size_t n_threads) {
  const size_t blocks = (n_threads + 255) / 256;
  return (int)std::min<size_t>(std::max<size_t>(blocks, 1), 256 * 16);
}

}  // namespace

size_t rope_table_floats(int S, int dh) { return (size_t)S * dh; }   // S * dh/2 (cos, sin) pairs

swarm_status rope_table(float* table, int S, int dh, hipStream_t st) {
  const int n = S * (dh / 2);
  hipLaunchKernelGGL(rope_table_kernel, dim3((n + 255) / 256), dim3(256), 0, st, (float2*)table, S, dh / 2);
  return launch_status();
}

swarm_status rope_apply(void* qkv, const float* table, int T, int S, int d, int dh, bool inverse, bool bf16,
                        hipStream_t st) {
  if (dh % 8 || d % dh) return SWARM_ERR_SHAPE;
  const int grid = stream_grid((size_t)T * (2 * d / 8));
  const float sign = inverse ? -1.0f : 1.0f;
  if (bf16)
    hipLaunchKernelGGL(rope_apply_kernel<bf16_raw>, dim3(grid), dim3(256), 0, st, (bf16_raw*)qkv,
                       (const float2*)table, T, S, d, dh, sign);
  else
    hipLaunchKernelGGL(rope_apply_kernel<float>, dim3(grid), dim3(256), 0, st, (float*)qkv, (const float2*)table, T, S,
                       d, dh, sign);
  return launch_status();
}

swarm_status geglu_fwd(const void* u, void* g, int T, int f, bool bf16, hipStream_t st) {
  if (f % 8) return SWARM_ERR_SHAPE;
  const int grid = stream_grid((size_t)T * (f / 8));
  if (bf16)
    hipLaunchKernelGGL(geglu_fwd_kernel<bf16_raw>, dim3(grid), dim3(256), 0, st, (const bf16_raw*)u, (bf16_raw*)g, T,
                       f);
  else
    hipLaunchKernelGGL(geglu_fwd_kernel<float>, dim3(grid), dim3(256), 0, st, (const float*)u, (float*)g, T, f);
  return launch_status();
}

swarm_status geglu_bwd(const void* dg, const void* u, void* du, int T, int f, bool bf16, hipStream_t st) {
  if (f % 8) return SWARM_ERR_SHAPE;
  const int grid = stream_grid((size_t)T * (f / 8));
  if (bf16)
    hipLaunchKernelGGL(geglu_bwd_kernel<bf16_raw>, dim3(grid), dim3(256), 0, st, (const bf16_raw*)dg,
                       (const bf16_raw*)u, (bf16_raw*)du, T, f);
  else
    hipLaunchKernelGGL(geglu_bwd_kernel<float>, dim3(grid), dim3(256), 0, st, (const float*)dg, (const float*)u,
                       (float*)du, T, f);
  return launch_status();
}

}  // namespace swarm
