// LAMB step for one parameter tensor (appendix "Additional Details for Section 4.3").  Three streaming kernels:
// moments + update direction + per-workgroup partial sums of |w|^2 and |u|^2; a single-workgroup, fixed-order
// reduction to the trust ratio; the weight update (and the copy in the stage's dtype).
#include <atomic>
#include <cmath>

#include "kernels.h"
#include "swarm_optim.h"

namespace swarm {
namespace {

constexpr int kThreads = 256;
constexpr int kPerThread = 16;                         // elements per thread in the first pass (4 x float4)
constexpr int kPerBlock = kThreads * kPerThread;

// Every element is touched once per pass, so all vector accesses are non-temporal: nothing is kept in the caches
// for a second use that never comes (5.2 -> 5.9 TB/s on the largest tensor).
typedef float f32x4n __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 ldg4(const float* p) {
  const f32x4n t = __builtin_nontemporal_load(reinterpret_cast<const f32x4n*>(p));
  return make_float4(t[0], t[1], t[2], t[3]);
}
__device__ __forceinline__ void stg4(float* p, const float4& v) {
  const f32x4n t = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(t, reinterpret_cast<f32x4n*>(p));
}

struct Hyper {
  float beta1, beta2, one_m_beta1, one_m_beta2, inv_bc1, inv_bc2, eps, wd, gscale, lr;
};

__global__ __launch_bounds__(kThreads) void lamb_moments_kernel(const float* __restrict__ w, const float* __restrict__ g,
                                                                float* __restrict__ m, float* __restrict__ v,
                                                                float* __restrict__ u, float* __restrict__ partial,
                                                                size_t n, Hyper h) {
  __shared__ float s_w[kThreads], s_u[kThreads];
  const size_t base = (size_t)blockIdx.x * kPerBlock;
  float sw = 0.f, su = 0.f;
#pragma unroll
  for (int it = 0; it < kPerThread / 4; ++it) {
    const size_t i = base + ((size_t)it * kThreads + threadIdx.x) * 4;
    if (i + 4 <= n) {
      const float4 w4 = ldg4(w + i), g4 = ldg4(g + i);
      float4 m4 = ldg4(m + i), v4 = ldg4(v + i), u4;
      const float wv[4] = {w4.x, w4.y, w4.z, w4.w}, gv[4] = {g4.x, g4.y, g4.z, g4.w};
      float mv[4] = {m4.x, m4.y, m4.z, m4.w}, vv[4] = {v4.x, v4.y, v4.z, v4.w}, uv[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float gs = gv[e] * h.gscale;
        mv[e] = h.beta1 * mv[e] + h.one_m_beta1 * gs;
        vv[e] = h.beta2 * vv[e] + h.one_m_beta2 * gs * gs;
        uv[e] = (mv[e] * h.inv_bc1) / (sqrtf(vv[e] * h.inv_bc2) + h.eps) + h.wd * wv[e];
        sw += wv[e] * wv[e];
        su += uv[e] * uv[e];
      }
      m4 = make_float4(mv[0], mv[1], mv[2], mv[3]); v4 = make_float4(vv[0], vv[1], vv[2], vv[3]);
      u4 = make_float4(uv[0], uv[1], uv[2], uv[3]);
      stg4(m + i, m4); stg4(v + i, v4);
      stg4(u + i, u4);
    } else {
      for (size_t j = i; j < n && j < i + 4; ++j) {          // ragged tail
        const float gs = g[j] * h.gscale;
        const float mj = h.beta1 * m[j] + h.one_m_beta1 * gs;
        const float vj = h.beta2 * v[j] + h.one_m_beta2 * gs * gs;
        const float uj = (mj * h.inv_bc1) / (sqrtf(vj * h.inv_bc2) + h.eps) + h.wd * w[j];
        m[j] = mj; v[j] = vj; u[j] = uj;
        sw += w[j] * w[j];
        su += uj * uj;
      }
    }
  }
  s_w[threadIdx.x] = sw; s_u[threadIdx.x] = su;
  __syncthreads();
  for (int k = kThreads / 2; k >= 1; k >>= 1) {
    if (threadIdx.x < k) { s_w[threadIdx.x] += s_w[threadIdx.x + k]; s_u[threadIdx.x] += s_u[threadIdx.x + k]; }
    __syncthreads();
  }
  if (threadIdx.x == 0) { partial[2 * (size_t)blockIdx.x] = s_w[0]; partial[2 * (size_t)blockIdx.x + 1] = s_u[0]; }
}

// ratio = |w| / |u| (1 if either is zero); doubles keep the long fixed-order sum accurate
__global__ __launch_bounds__(kThreads) void lamb_ratio_kernel(const float* __restrict__ partial, size_t nblocks,
                                                              float* __restrict__ ratio_out, float* __restrict__ user) {
  __shared__ double s_w[kThreads], s_u[kThreads];
  double sw = 0.0, su = 0.0;
  for (size_t b = threadIdx.x; b < nblocks; b += kThreads) { sw += partial[2 * b]; su += partial[2 * b + 1]; }
  s_w[threadIdx.x] = sw; s_u[threadIdx.x] = su;
  __syncthreads();
  for (int k = kThreads / 2; k >= 1; k >>= 1) {
    if (threadIdx.x < k) { s_w[threadIdx.x] += s_w[threadIdx.x + k]; s_u[threadIdx.x] += s_u[threadIdx.x + k]; }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const double nw = sqrt(s_w[0]), nu = sqrt(s_u[0]);
    const float r = (nw > 0.0 && nu > 0.0) ? (float)(nw / nu) : 1.0f;
    *ratio_out = r;
    if (user) *user = r;
  }
}

template <typename T>
__global__ __launch_bounds__(kThreads) void lamb_apply_kernel(float* __restrict__ w, const float* __restrict__ u,
                                                              T* __restrict__ param, const float* __restrict__ ratio,
                                                              size_t n, float lr) {
  const float step = lr * *ratio;
  const size_t n4 = n / 4;
  constexpr int U = kPerThread / 4;
  const size_t i0 = (size_t)blockIdx.x * (kThreads * U) + threadIdx.x;
  float4 x[U], d[U];
#pragma unroll
  for (int it = 0; it < U; ++it) {
    const size_t i = i0 + (size_t)it * kThreads;
    if (i < n4) { x[it] = ldg4(w + 4 * i); d[it] = ldg4(u + 4 * i); }
  }
#pragma unroll
  for (int it = 0; it < U; ++it) {
    const size_t i = i0 + (size_t)it * kThreads;
    if (i >= n4) continue;
    float4 y = x[it];
    y.x -= step * d[it].x; y.y -= step * d[it].y; y.z -= step * d[it].z; y.w -= step * d[it].w;
    stg4(w + 4 * i, y);
    if (param) {
      if constexpr (sizeof(T) == 4) {
        reinterpret_cast<float4*>(param)[i] = y;
      } else {
        T r[4];
        Elem<T>::store(r, y.x); Elem<T>::store(r + 1, y.y); Elem<T>::store(r + 2, y.z); Elem<T>::store(r + 3, y.w);
        reinterpret_cast<uint2*>(param)[i] = *reinterpret_cast<const uint2*>(r);
      }
    }
  }
  if (blockIdx.x == 0 && threadIdx.x < n - n4 * 4) {           // ragged tail
    const size_t i = n4 * 4 + threadIdx.x;
    const float x = w[i] - step * u[i];
    w[i] = x;
    if (param) Elem<T>::store(param + i, x);
  }
}

size_t n_blocks(size_t n) { return (n + kPerBlock - 1) / kPerBlock; }

}  // namespace
}  // namespace swarm

using namespace swarm;

// Scratch of swarm_lamb_step_static: the update direction of the largest tensor it accepts, the partial sums of
// its norms and the ratio.  One copy per GPU, at an address of its own, held until the process ends.
constexpr size_t kStaticU = SWARM_LAMB_STATIC_MAX_ELEMS * sizeof(float);
constexpr size_t kStaticPartial = (SWARM_LAMB_STATIC_MAX_ELEMS / kPerBlock) * 2 * sizeof(float);
static_assert(SWARM_LAMB_STATIC_MAX_ELEMS % kPerBlock == 0 && kStaticU % 256 == 0 && kStaticPartial % 256 == 0, "");
static __device__ __align__(256) unsigned char scratch[kStaticU + kStaticPartial + 256];

extern "C" size_t swarm_lamb_workspace_bytes(size_t n_elems) {
  if (n_elems < 1) return 0;
  const size_t u = (n_elems * 4 + 255) & ~(size_t)255;
  const size_t p = (n_blocks(n_elems) * 8 + 255) & ~(size_t)255;
  return u + p + 256;
}

namespace swarm {
namespace {

// The three launches of one update; u [n] fp32, partial [2 * n_blocks(n)] fp32 and ratio [1] fp32 are scratch that
// the kernels overwrite before they read it (nothing has to be cleared between calls).
swarm_status lamb_launch(const swarm_lamb_config* cfg, size_t n, float* master, void* param, int32_t dtype,
                         const float* grad, float* m, float* v, float* trust_ratio, float* u, float* partial,
                         float* ratio, hipStream_t st) {
  const size_t nb = n_blocks(n);
  Hyper h;
  h.beta1 = cfg->beta1; h.beta2 = cfg->beta2; h.one_m_beta1 = 1.0f - cfg->beta1; h.one_m_beta2 = 1.0f - cfg->beta2;
  h.inv_bc1 = (float)(1.0 / (1.0 - std::pow((double)cfg->beta1, (double)cfg->step)));
  h.inv_bc2 = (float)(1.0 / (1.0 - std::pow((double)cfg->beta2, (double)cfg->step)));
  h.eps = cfg->eps; h.wd = cfg->weight_decay; h.gscale = cfg->grad_scale; h.lr = cfg->lr;
  hipLaunchKernelGGL(lamb_moments_kernel, dim3((unsigned)nb), dim3(kThreads), 0, st, master, grad, m, v, u, partial, n, h);
  hipLaunchKernelGGL(lamb_ratio_kernel, dim3(1), dim3(kThreads), 0, st, partial, nb, ratio, trust_ratio);
  const unsigned grid = (unsigned)nb;   // one workgroup per kPerBlock elements, as in the first pass
  if (param && dtype == SWARM_BF16)
    hipLaunchKernelGGL(lamb_apply_kernel<bf16_raw>, dim3(grid), dim3(kThreads), 0, st, master, u, (bf16_raw*)param,
                       ratio, n, cfg->lr);
  else
    hipLaunchKernelGGL(lamb_apply_kernel<float>, dim3(grid), dim3(kThreads), 0, st, master, u, (float*)param, ratio, n,
                       cfg->lr);
  return launch_status();
}

swarm_status lamb_check(const swarm_lamb_config* cfg, size_t n, const float* master, const void* param, int32_t dtype,
                        const float* grad, const float* m, const float* v) {
  if (!cfg || !master || !grad || !m || !v) return SWARM_ERR_NULL;
  if (param && dtype != SWARM_F32 && dtype != SWARM_BF16) return SWARM_ERR_DTYPE;
  if (n < 1 || cfg->step < 1 || !(cfg->beta1 >= 0.f && cfg->beta1 < 1.f) || !(cfg->beta2 >= 0.f && cfg->beta2 < 1.f) ||
      !(cfg->eps > 0.f) || !(cfg->lr >= 0.f) || !(cfg->weight_decay >= 0.f))
    return SWARM_ERR_SHAPE;
  auto al16 = [](const void* q) { return ((uintptr_t)q & 15) == 0; };
  if (!al16(master) || !al16(grad) || !al16(m) || !al16(v) || !al16(param)) return SWARM_ERR_SHAPE;
  return SWARM_OK;
}

// Device address of `scratch` on the current device (looked up once per device; the array's name is only a
// host-side handle and is never passed to a kernel).
std::atomic<unsigned char*> g_scratch_ptr[kMaxDevices];
unsigned char* static_scratch() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  unsigned char* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    void* q = nullptr;
    if (hipGetSymbolAddress(&q, HIP_SYMBOL(scratch)) != hipSuccess || !q) return nullptr;
    p = (unsigned char*)q;
    g_scratch_ptr[dev].store(p, std::memory_order_release);
  }
  return p;
}

}  // namespace
}  // namespace swarm

extern "C" swarm_status swarm_lamb_step(const swarm_lamb_config* cfg, size_t n, float* master, void* param,
                                        int32_t dtype, const float* grad, float* m, float* v, float* trust_ratio,
                                        void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!workspace) return SWARM_ERR_NULL;
  const swarm_status chk = lamb_check(cfg, n, master, param, dtype, grad, m, v);
  if (chk != SWARM_OK) return chk;
  if ((uintptr_t)workspace & 255) return SWARM_ERR_SHAPE;
  if (swarm_lamb_workspace_bytes(n) > workspace_bytes) return SWARM_ERR_WORKSPACE;
  float* u = (float*)workspace;
  float* partial = (float*)((char*)workspace + ((n * 4 + 255) & ~(size_t)255));
  const size_t nb = n_blocks(n);
  float* ratio = partial + 2 * nb + (64 - (2 * nb) % 64) % 64;   // behind the partial sums, inside the slack
  return lamb_launch(cfg, n, master, param, dtype, grad, m, v, trust_ratio, u, partial, ratio, (hipStream_t)hip_stream);
}

extern "C" swarm_status swarm_lamb_step_static(const swarm_lamb_config* cfg, size_t n, float* master, void* param,
                                               int32_t dtype, const float* grad, float* m, float* v,
                                               float* trust_ratio, void* hip_stream) {
  const swarm_status chk = lamb_check(cfg, n, master, param, dtype, grad, m, v);
  if (chk != SWARM_OK) return chk;
  if (n > SWARM_LAMB_STATIC_MAX_ELEMS) return SWARM_ERR_WORKSPACE;
  unsigned char* base = static_scratch();
  if (!base) return SWARM_ERR_LAUNCH;
  return lamb_launch(cfg, n, master, param, dtype, grad, m, v, trust_ratio, (float*)base, (float*)(base + kStaticU),
                     (float*)(base + kStaticU + kStaticPartial), (hipStream_t)hip_stream);
}
