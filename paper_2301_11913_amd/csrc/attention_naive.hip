// Direct (one query row or one key row per workgroup) causal attention in fp32 arithmetic.
// Used by the fp32 parity configuration and for shapes the MFMA kernels do not cover.
// Deterministic: every sum runs in a fixed order.
#include "kernels.h"

namespace swarm {
namespace {

constexpr int kNT = 256;

__device__ __forceinline__ float block_reduce(float v, bool is_max, float* red) {
  v = is_max ? wave_max(v) : wave_sum(v);
  const int wave = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[wave] = v;
  __syncthreads();
  float r = red[0];
  for (int w = 1; w < kNT / 64; ++w) r = is_max ? fmaxf(r, red[w]) : r + red[w];
  return r;
}

// grid (S, H, B).  LDS: q[dh] + s[S] floats.
template <typename T>
__global__ __launch_bounds__(kNT) void attn_fwd_naive_kernel(const T* __restrict__ qkv, T* __restrict__ o,
                                                             float* __restrict__ lse, int S, int H, int dh) {
  extern __shared__ float sm[];
  __shared__ float red[kNT / 64];
  float* qs = sm;
  float* sc = sm + dh;
  const int i = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int d = H * dh, ld = 3 * d;
  const T* base = qkv + (size_t)b * S * ld + h * dh;
  const float scale = 1.0f / sqrtf((float)dh);
  for (int c = threadIdx.x; c < dh; c += kNT) qs[c] = Elem<T>::load(base + (size_t)i * ld + c);
  __syncthreads();
  float mx = -INFINITY;
  for (int j = threadIdx.x; j <= i; j += kNT) {
    const T* kr = base + (size_t)j * ld + d;
    float s = 0.f;
    for (int c = 0; c < dh; ++c) s = fmaf(qs[c], Elem<T>::load(kr + c), s);
    s *= scale;
    sc[j] = s;
    mx = fmaxf(mx, s);
  }
  mx = block_reduce(mx, true, red);
  float sum = 0.f;
  for (int j = threadIdx.x; j <= i; j += kNT) {
    const float e = expf(sc[j] - mx);
    sc[j] = e;
    sum += e;
  }
  sum = block_reduce(sum, false, red);
  const float inv = 1.0f / sum;
  for (int c = threadIdx.x; c < dh; c += kNT) {
    float acc = 0.f;
    for (int j = 0; j <= i; ++j) acc = fmaf(sc[j], Elem<T>::load(base + (size_t)j * ld + 2 * d + c), acc);
    Elem<T>::store(o + ((size_t)b * S + i) * d + h * dh + c, acc * inv);
  }
  if (threadIdx.x == 0) lse[((size_t)b * H + h) * S + i] = mx + logf(sum);
}

// delta[b,h,i] = sum_c do[i,c] * o[i,c].  grid (S, H, B), one wavefront.
template <typename T>
__global__ __launch_bounds__(64) void attn_delta_kernel(const T* __restrict__ o, const T* __restrict__ dout,
                                                        float* __restrict__ delta, int S, int H, int dh) {
  const int i = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const size_t off = ((size_t)b * S + i) * H * dh + h * dh;
  float s = 0.f;
  for (int c = threadIdx.x; c < dh; c += 64) s += Elem<T>::load(o + off + c) * Elem<T>::load(dout + off + c);
  s = wave_sum(s);
  if (threadIdx.x == 0) delta[((size_t)b * H + h) * S + i] = s;
}

// dq for one query row.  grid (S, H, B).  LDS: q[dh] + do[dh] + ds[S].
template <typename T>
__global__ __launch_bounds__(kNT) void attn_bwd_dq_naive_kernel(const T* __restrict__ qkv, const T* __restrict__ dout,
                                                                const float* __restrict__ lse,
                                                                const float* __restrict__ delta,
                                                                T* __restrict__ dqkv, int S, int H, int dh) {
  extern __shared__ float sm[];
  float* qs = sm;
  float* dos = sm + dh;
  float* ds = sm + 2 * dh;
  const int i = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int d = H * dh, ld = 3 * d;
  const T* base = qkv + (size_t)b * S * ld + h * dh;
  const float scale = 1.0f / sqrtf((float)dh);
  for (int c = threadIdx.x; c < dh; c += kNT) {
    qs[c] = Elem<T>::load(base + (size_t)i * ld + c);
    dos[c] = Elem<T>::load(dout + ((size_t)b * S + i) * d + h * dh + c);
  }
  __syncthreads();
  const float L = lse[((size_t)b * H + h) * S + i];
  const float dl = delta[((size_t)b * H + h) * S + i];
  for (int j = threadIdx.x; j <= i; j += kNT) {
    const T* kr = base + (size_t)j * ld + d;
    const T* vr = base + (size_t)j * ld + 2 * d;
    float s = 0.f, dp = 0.f;
    for (int c = 0; c < dh; ++c) {
      s = fmaf(qs[c], Elem<T>::load(kr + c), s);
      dp = fmaf(dos[c], Elem<T>::load(vr + c), dp);
    }
    const float p = expf(s * scale - L);
    ds[j] = p * (dp - dl);
  }
  __syncthreads();
  for (int c = threadIdx.x; c < dh; c += kNT) {
    float acc = 0.f;
    for (int j = 0; j <= i; ++j) acc = fmaf(ds[j], Elem<T>::load(base + (size_t)j * ld + d + c), acc);
    Elem<T>::store(dqkv + ((size_t)b * S + i) * ld + h * dh + c, acc * scale);
  }
}

// dk, dv for one key row j.  grid (S, H, B).  LDS: k[dh] + v[dh] + p[S] + ds[S].
template <typename T>
__global__ __launch_bounds__(kNT) void attn_bwd_dkdv_naive_kernel(const T* __restrict__ qkv,
                                                                  const T* __restrict__ dout,
                                                                  const float* __restrict__ lse,
                                                                  const float* __restrict__ delta,
                                                                  T* __restrict__ dqkv, int S, int H, int dh) {
  extern __shared__ float sm[];
  float* ks = sm;
  float* vs = sm + dh;
  float* ps = sm + 2 * dh;
  float* ds = ps + S;
  const int j = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int d = H * dh, ld = 3 * d;
  const T* base = qkv + (size_t)b * S * ld + h * dh;
  const float scale = 1.0f / sqrtf((float)dh);
  for (int c = threadIdx.x; c < dh; c += kNT) {
    ks[c] = Elem<T>::load(base + (size_t)j * ld + d + c);
    vs[c] = Elem<T>::load(base + (size_t)j * ld + 2 * d + c);
  }
  __syncthreads();
  for (int i = j + threadIdx.x; i < S; i += kNT) {
    const T* qr = base + (size_t)i * ld;
    const T* dor = dout + ((size_t)b * S + i) * d + h * dh;
    float s = 0.f, dp = 0.f;
    for (int c = 0; c < dh; ++c) {
      s = fmaf(Elem<T>::load(qr + c), ks[c], s);
      dp = fmaf(Elem<T>::load(dor + c), vs[c], dp);
    }
    const size_t r = ((size_t)b * H + h) * S + i;
    const float p = expf(s * scale - lse[r]);
    ps[i] = p;
    ds[i] = p * (dp - delta[r]);
  }
  __syncthreads();
  for (int c = threadIdx.x; c < dh; c += kNT) {
    float av = 0.f, ak = 0.f;
    for (int i = j; i < S; ++i) {
      av = fmaf(ps[i], Elem<T>::load(dout + ((size_t)b * S + i) * d + h * dh + c), av);
      ak = fmaf(ds[i], Elem<T>::load(base + (size_t)i * ld + c), ak);
    }
    Elem<T>::store(dqkv + ((size_t)b * S + j) * ld + d + h * dh + c, ak * scale);
    Elem<T>::store(dqkv + ((size_t)b * S + j) * ld + 2 * d + h * dh + c, av);
  }
}

template <typename T>
swarm_status fwd_t(const T* qkv, T* o, float* lse, int B, int S, int H, int dh, hipStream_t st) {
  const size_t lds = (size_t)(dh + S) * sizeof(float);
  if (lds > 60 * 1024) return SWARM_ERR_SHAPE;
  hipLaunchKernelGGL(attn_fwd_naive_kernel<T>, dim3(S, H, B), dim3(kNT), lds, st, qkv, o, lse, S, H, dh);
  return launch_status();
}

template <typename T>
swarm_status bwd_t(const T* qkv, const T* o, const T* dout, const float* lse, float* delta, T* dqkv, int B, int S,
                   int H, int dh, hipStream_t st) {
  const size_t lds = (size_t)(2 * dh + 2 * S) * sizeof(float);
  if (lds > 60 * 1024) return SWARM_ERR_SHAPE;
  hipLaunchKernelGGL(attn_delta_kernel<T>, dim3(S, H, B), dim3(64), 0, st, o, dout, delta, S, H, dh);
  hipLaunchKernelGGL(attn_bwd_dq_naive_kernel<T>, dim3(S, H, B), dim3(kNT), (size_t)(2 * dh + S) * sizeof(float),
                     st, qkv, dout, lse, delta, dqkv, S, H, dh);
  hipLaunchKernelGGL(attn_bwd_dkdv_naive_kernel<T>, dim3(S, H, B), dim3(kNT), lds, st, qkv, dout, lse, delta, dqkv,
                     S, H, dh);
  return launch_status();
}

}  // namespace

swarm_status attention_fwd_naive(const void* qkv, void* o, float* lse, int B, int S, int H, int dh, bool bf16,
                                 hipStream_t st) {
  if (bf16) return fwd_t<bf16_raw>((const bf16_raw*)qkv, (bf16_raw*)o, lse, B, S, H, dh, st);
  return fwd_t<float>((const float*)qkv, (float*)o, lse, B, S, H, dh, st);
}

swarm_status attention_bwd_naive(const void* qkv, const void* o, const void* dout, const float* lse, float* delta,
                                 void* dqkv, int B, int S, int H, int dh, bool bf16, hipStream_t st) {
  if (bf16)
    return bwd_t<bf16_raw>((const bf16_raw*)qkv, (const bf16_raw*)o, (const bf16_raw*)dout, lse, delta,
                           (bf16_raw*)dqkv, B, S, H, dh, st);
  return bwd_t<float>((const float*)qkv, (const float*)o, (const float*)dout, lse, delta, (float*)dqkv, B, S, H, dh,
                      st);
}

}  // namespace swarm
