// LayerNorm forward/backward and column-sum reductions: streaming, HBM-bound kernels.
//
// One wavefront owns one token row at a time.  A lane owns 8-element chunks
// l, l+64, ... of the row (16-byte loads for bf16, 2 x 16 bytes for fp32), keeps
// them in registers, and the row statistics are 64-lane butterfly reductions.
// Parameter-gradient reductions are two-stage and fixed-order (no atomics), so
// results are bitwise reproducible.
#include "kernels.h"

namespace swarm {

namespace {

constexpr int kLnThreads = 256;              // 4 wavefronts per workgroup
constexpr int kLnWaves = kLnThreads / kWave;
constexpr int kLnRowsPerBlock = 16;          // backward: rows per workgroup

template <typename T> struct V8;
template <> struct V8<bf16_raw> {
  static __device__ __forceinline__ void load(const bf16_raw* p, float (&x)[8]) {
    uint4 v = *reinterpret_cast<const uint4*>(p);
    uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      x[2 * i] = __uint_as_float(w[i] << 16);
      x[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
    }
  }
  static __device__ __forceinline__ void store(bf16_raw* p, const float (&x)[8]) {
    uint4 v;
    v.x = pack_bf16x2(x[0], x[1]); v.y = pack_bf16x2(x[2], x[3]);
    v.z = pack_bf16x2(x[4], x[5]); v.w = pack_bf16x2(x[6], x[7]);
    *reinterpret_cast<uint4*>(p) = v;
  }
};
template <> struct V8<float> {
  static __device__ __forceinline__ void load(const float* p, float (&x)[8]) {
    float4 a = *reinterpret_cast<const float4*>(p);
    float4 b = *reinterpret_cast<const float4*>(p + 4);
    x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
  }
  static __device__ __forceinline__ void store(float* p, const float (&x)[8]) {
    *reinterpret_cast<float4*>(p) = make_float4(x[0], x[1], x[2], x[3]);
    *reinterpret_cast<float4*>(p + 4) = make_float4(x[4], x[5], x[6], x[7]);
  }
};

// NIT = chunks per lane held in registers (d <= NIT * 512).
template <typename T, int NIT>
__global__ __launch_bounds__(kLnThreads) void ln_fwd_kernel(const T* __restrict__ x, const T* __restrict__ gamma,
                                                            const T* __restrict__ beta, T* __restrict__ y,
                                                            float* __restrict__ mean, float* __restrict__ rstd,
                                                            int rows, int d, float eps) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int nchunk = d >> 3;
  const float inv_d = 1.0f / (float)d;
  for (int row = blockIdx.x * kLnWaves + wave; row < rows; row += gridDim.x * kLnWaves) {
    const T* xr = x + (size_t)row * d;
    float v[NIT][8];
    float s = 0.f;
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int c = lane + it * 64;
      if (c < nchunk) {
        V8<T>::load(xr + c * 8, v[it]);
#pragma unroll
        for (int i = 0; i < 8; ++i) s += v[it][i];
      }
    }
    const float mu = wave_sum(s) * inv_d;
    float q = 0.f;
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int c = lane + it * 64;
      if (c < nchunk) {
#pragma unroll
        for (int i = 0; i < 8; ++i) { const float t = v[it][i] - mu; q += t * t; }
      }
    }
    const float var = wave_sum(q) * inv_d;
    const float r = 1.0f / sqrtf(var + eps);
    T* yr = y + (size_t)row * d;
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int c = lane + it * 64;
      if (c < nchunk) {
        float g[8], b[8], o[8];
        V8<T>::load(gamma + c * 8, g);
        V8<T>::load(beta + c * 8, b);
#pragma unroll
        for (int i = 0; i < 8; ++i) o[i] = (v[it][i] - mu) * r * g[i] + b[i];
        V8<T>::store(yr + c * 8, o);
      }
    }
    if (lane == 0) { mean[row] = mu; rstd[row] = r; }
  }
}

// Backward.  Each wavefront walks kLnRowsPerBlock / 4 rows, keeps per-lane partial sums of
// dgamma / dbeta, and the four wavefronts combine them through LDS in wave order.
// partial: [gridDim.x][2][d] floats (dgamma then dbeta).
template <typename T, int NIT>
__global__ __launch_bounds__(kLnThreads) void ln_bwd_kernel(const T* __restrict__ dy, const T* __restrict__ x,
                                                            const float* __restrict__ mean,
                                                            const float* __restrict__ rstd,
                                                            const T* __restrict__ gamma, const T* __restrict__ dres,
                                                            T* __restrict__ dx, float* __restrict__ partial, int rows,
                                                            int d) {
  extern __shared__ float lds_part[];          // [2][d]
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int nchunk = d >> 3;
  const float inv_d = 1.0f / (float)d;
  float g[NIT][8], pg[NIT][8], pb[NIT][8];
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    const int c = lane + it * 64;
#pragma unroll
    for (int i = 0; i < 8; ++i) { pg[it][i] = 0.f; pb[it][i] = 0.f; g[it][i] = 0.f; }
    if (c < nchunk) V8<T>::load(gamma + c * 8, g[it]);
  }
  const int row0 = blockIdx.x * kLnRowsPerBlock;
  for (int rr = wave; rr < kLnRowsPerBlock; rr += kLnWaves) {
    const int row = row0 + rr;
    if (row >= rows) break;
    const float mu = mean[row], r = rstd[row];
    float xh[NIT][8], t[NIT][8];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int c = lane + it * 64;
      if (c < nchunk) {
        float xv[8], dv[8];
        V8<T>::load(x + (size_t)row * d + c * 8, xv);
        V8<T>::load(dy + (size_t)row * d + c * 8, dv);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          xh[it][i] = (xv[i] - mu) * r;
          t[it][i] = dv[i] * g[it][i];
          s1 += t[it][i];
          s2 += t[it][i] * xh[it][i];
          pg[it][i] += dv[i] * xh[it][i];
          pb[it][i] += dv[i];
        }
      }
    }
    const float m1 = wave_sum(s1) * inv_d;
    const float m2 = wave_sum(s2) * inv_d;
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int c = lane + it * 64;
      if (c < nchunk) {
        float rs[8], o[8];
        V8<T>::load(dres + (size_t)row * d + c * 8, rs);
#pragma unroll
        for (int i = 0; i < 8; ++i) o[i] = rs[i] + r * (t[it][i] - m1 - xh[it][i] * m2);
        V8<T>::store(dx + (size_t)row * d + c * 8, o);
      }
    }
  }
  // fixed-order combine: wave 0 stores, waves 1..3 add in turn
  for (int w = 0; w < kLnWaves; ++w) {
    if (wave == w) {
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        const int c = lane + it * 64;
        if (c < nchunk) {
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            if (w == 0) {
              lds_part[c * 8 + i] = pg[it][i];
              lds_part[d + c * 8 + i] = pb[it][i];
            } else {
              lds_part[c * 8 + i] += pg[it][i];
              lds_part[d + c * 8 + i] += pb[it][i];
            }
          }
        }
      }
    }
    __syncthreads();
  }
  float* out = partial + (size_t)blockIdx.x * 2 * d;
  for (int i = threadIdx.x; i < 2 * d; i += kLnThreads) out[i] = lds_part[i];
}

// Stage 1 of a column sum: workgroup = 64 column chunks (512 columns) x 4 row groups over kCsRows rows.
constexpr int kCsRows = 128;
template <typename T>
__global__ __launch_bounds__(256) void colsum_partial_kernel(const T* __restrict__ X, int rows, int N,
                                                             float* __restrict__ partial) {
  __shared__ float red[4][512];
  const int cchunk = blockIdx.x * 64 + (threadIdx.x & 63);
  const int rg = threadIdx.x >> 6;
  const int r0 = blockIdx.y * kCsRows;
  const int r1 = min(rows, r0 + kCsRows);
  float acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = 0.f;
  const bool active = cchunk * 8 < N;
  if (active) {
    for (int r = r0 + rg; r < r1; r += 4) {
      float v[8];
      V8<T>::load(X + (size_t)r * N + cchunk * 8, v);
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] += v[i];
    }
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) red[rg][(threadIdx.x & 63) * 8 + i] = acc[i];
  __syncthreads();
  for (int c = threadIdx.x; c < 512; c += 256) {
    const int col = blockIdx.x * 512 + c;
    if (col < N) partial[(size_t)blockIdx.y * N + col] = ((red[0][c] + red[1][c]) + red[2][c]) + red[3][c];
  }
}

// Stage 2: out[c] += sum_p partial[p*stride + c], p ascending.  Workgroup = 64 columns x 4 row groups.
__global__ __launch_bounds__(256) void reduce_rows_accum_kernel(const float* __restrict__ partial, int P, int C,
                                                                size_t stride, float* __restrict__ out) {
  __shared__ float red[4][64];
  const int c = blockIdx.x * 64 + (threadIdx.x & 63);
  const int rg = threadIdx.x >> 6;
  const int per = (P + 3) / 4;
  const int p0 = rg * per, p1 = min(P, p0 + per);
  float s = 0.f;
  if (c < C)
    for (int p = p0; p < p1; ++p) s += partial[(size_t)p * stride + c];
  red[rg][threadIdx.x & 63] = s;
  __syncthreads();
  if (rg == 0 && c < C) {
    const int l = threadIdx.x & 63;
    out[c] += ((red[0][l] + red[1][l]) + red[2][l]) + red[3][l];
  }
}

template <typename T>
swarm_status ln_fwd_dispatch(const T* x, const T* g, const T* b, T* y, float* mean, float* rstd, int rows, int d,
                             float eps, hipStream_t st) {
  const int grid = std::min((rows + kLnWaves - 1) / kLnWaves, 256 * 8);
#define LN_FWD(NIT)                                                                                         \
  hipLaunchKernelGGL((ln_fwd_kernel<T, NIT>), dim3(grid), dim3(kLnThreads), 0, st, x, g, b, y, mean, rstd, \
                     rows, d, eps)
  if (d <= 512) LN_FWD(1);
  else if (d <= 1024) LN_FWD(2);
  else if (d <= 2048) LN_FWD(4);
  else if (d <= 4096) LN_FWD(8);
  else if (d <= 8192) LN_FWD(16);
  else return SWARM_ERR_SHAPE;
#undef LN_FWD
  return launch_status();
}

template <typename T>
swarm_status ln_bwd_dispatch(const T* dy, const T* x, const float* mean, const float* rstd, const T* g,
                             const T* dres, T* dx, float* partial, int rows, int d, hipStream_t st) {
  const int grid = (rows + kLnRowsPerBlock - 1) / kLnRowsPerBlock;
  const size_t lds = (size_t)2 * d * sizeof(float);
#define LN_BWD(NIT)                                                                                          \
  hipLaunchKernelGGL((ln_bwd_kernel<T, NIT>), dim3(grid), dim3(kLnThreads), lds, st, dy, x, mean, rstd, g, \
                     dres, dx, partial, rows, d)
  if (d <= 512) LN_BWD(1);
  else if (d <= 1024) LN_BWD(2);
  else if (d <= 2048) LN_BWD(4);
  else if (d <= 4096) LN_BWD(8);
  else if (d <= 8192) LN_BWD(16);
  else return SWARM_ERR_SHAPE;
#undef LN_BWD
  return launch_status();
}

}  // namespace

swarm_status layernorm_fwd(const void* x, const void* gamma, const void* beta, void* y, float* mean, float* rstd,
                           int T, int d, float eps, bool bf16, hipStream_t st) {
  if (bf16)
    return ln_fwd_dispatch<bf16_raw>((const bf16_raw*)x, (const bf16_raw*)gamma, (const bf16_raw*)beta,
                                     (bf16_raw*)y, mean, rstd, T, d, eps, st);
  return ln_fwd_dispatch<float>((const float*)x, (const float*)gamma, (const float*)beta, (float*)y, mean, rstd,
                                T, d, eps, st);
}

size_t layernorm_bwd_scratch_floats(int T, int d) {
  return (size_t)((T + kLnRowsPerBlock - 1) / kLnRowsPerBlock) * 2 * d;
}

swarm_status layernorm_bwd(const void* dy, const void* x, const float* mean, const float* rstd, const void* gamma,
                           const void* dres, void* dx, float* dgamma, float* dbeta, float* partial, int T, int d,
                           bool bf16, hipStream_t st) {
  swarm_status s;
  if (bf16)
    s = ln_bwd_dispatch<bf16_raw>((const bf16_raw*)dy, (const bf16_raw*)x, mean, rstd, (const bf16_raw*)gamma,
                                  (const bf16_raw*)dres, (bf16_raw*)dx, partial, T, d, st);
  else
    s = ln_bwd_dispatch<float>((const float*)dy, (const float*)x, mean, rstd, (const float*)gamma,
                               (const float*)dres, (float*)dx, partial, T, d, st);
  if (s != SWARM_OK) return s;
  const int P = (T + kLnRowsPerBlock - 1) / kLnRowsPerBlock;
  const int grid = (d + 63) / 64;
  hipLaunchKernelGGL(reduce_rows_accum_kernel, dim3(grid), dim3(256), 0, st, partial, P, d, (size_t)2 * d, dgamma);
  hipLaunchKernelGGL(reduce_rows_accum_kernel, dim3(grid), dim3(256), 0, st, partial + d, P, d, (size_t)2 * d,
                     dbeta);
  return launch_status();
}

size_t colsum_scratch_floats(int T, int N) { return (size_t)((T + kCsRows - 1) / kCsRows) * N; }

swarm_status colsum_accum(const void* X, int T, int N, float* out, float* partial, bool bf16, hipStream_t st) {
  const int P = (T + kCsRows - 1) / kCsRows;
  dim3 grid((N + 511) / 512, P);
  if (bf16)
    hipLaunchKernelGGL(colsum_partial_kernel<bf16_raw>, grid, dim3(256), 0, st, (const bf16_raw*)X, T, N, partial);
  else
    hipLaunchKernelGGL(colsum_partial_kernel<float>, grid, dim3(256), 0, st, (const float*)X, T, N, partial);
  hipLaunchKernelGGL(reduce_rows_accum_kernel, dim3((N + 63) / 64), dim3(256), 0, st, partial, P, N, (size_t)N,
                     out);
  return launch_status();
}

}  // namespace swarm
