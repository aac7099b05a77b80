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
// backward: rows per workgroup (a multiple of the rows per barrier); fewer for short inputs, so that the launch
// still has at least two workgroups per compute unit
static inline int ln_rows_per_block(int T) { return T >= 8192 ? 16 : T >= 4096 ? 8 : 4; }

template <typename T> struct V8;
template <> struct V8<bf16_raw> {
  struct Raw { uint4 v; };                   // 8 elements as loaded (keeps register use low)
  static __device__ __forceinline__ float rounded(float x) { return bf16_bits_to_float(float_to_bf16_bits(x)); }
  static __device__ __forceinline__ Raw load_raw(const bf16_raw* p) { return Raw{*reinterpret_cast<const uint4*>(p)}; }
  static __device__ __forceinline__ Raw make_raw(const float (&x)[8]) {
    return Raw{make_uint4(pack_bf16x2(x[0], x[1]), pack_bf16x2(x[2], x[3]), pack_bf16x2(x[4], x[5]),
                          pack_bf16x2(x[6], x[7]))};
  }
  static __device__ __forceinline__ void unpack(const Raw& r, float (&x)[8]) {
    const uint32_t w[4] = {r.v.x, r.v.y, r.v.z, r.v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      x[2 * i] = __uint_as_float(w[i] << 16);
      x[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
    }
  }
  // the compiler may not carry anything computed from r across this point (keeps the unpacked copy out of registers)
  static __device__ __forceinline__ void opaque(Raw& r) {
    asm volatile("" : "+v"(r.v.x), "+v"(r.v.y), "+v"(r.v.z), "+v"(r.v.w));
  }
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
  struct Raw { float4 a, b; };
  static __device__ __forceinline__ float rounded(float x) { return x; }
  static __device__ __forceinline__ Raw load_raw(const float* p) {
    return Raw{*reinterpret_cast<const float4*>(p), *reinterpret_cast<const float4*>(p + 4)};
  }
  static __device__ __forceinline__ Raw make_raw(const float (&x)[8]) {
    return Raw{make_float4(x[0], x[1], x[2], x[3]), make_float4(x[4], x[5], x[6], x[7])};
  }
  static __device__ __forceinline__ void unpack(const Raw& r, float (&x)[8]) {
    x[0] = r.a.x; x[1] = r.a.y; x[2] = r.a.z; x[3] = r.a.w; x[4] = r.b.x; x[5] = r.b.y; x[6] = r.b.z; x[7] = r.b.w;
  }
  static __device__ __forceinline__ void opaque(Raw&) {}      // fp32: the raw form is the unpacked form
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

// n = 1, 2 or 4 consecutive elements of type T from floats (the maxout outputs of one 8-element chunk)
template <typename T, int N>
__device__ __forceinline__ void store_small(T* p, const float (&x)[8]) {
  if constexpr (sizeof(T) == 2) {
    if constexpr (N == 4) *reinterpret_cast<uint2*>(p) = make_uint2(pack_bf16x2(x[0], x[1]), pack_bf16x2(x[2], x[3]));
    else if constexpr (N == 2) *reinterpret_cast<uint32_t*>(p) = pack_bf16x2(x[0], x[1]);
    else *p = (T)float_to_bf16_bits(x[0]);
  } else {
    if constexpr (N == 4) *reinterpret_cast<float4*>(p) = make_float4(x[0], x[1], x[2], x[3]);
    else if constexpr (N == 2) *reinterpret_cast<float2*>(p) = make_float2(x[0], x[1]);
    else *p = x[0];
  }
}
template <typename T, int N>
__device__ __forceinline__ void load_small(const T* p, float (&x)[8]) {
  if constexpr (sizeof(T) == 2) {
    if constexpr (N == 4) {
      const uint2 v = *reinterpret_cast<const uint2*>(p);
      x[0] = __uint_as_float(v.x << 16); x[1] = __uint_as_float(v.x & 0xFFFF0000u);
      x[2] = __uint_as_float(v.y << 16); x[3] = __uint_as_float(v.y & 0xFFFF0000u);
    } else if constexpr (N == 2) {
      const uint32_t v = *reinterpret_cast<const uint32_t*>(p);
      x[0] = __uint_as_float(v << 16); x[1] = __uint_as_float(v & 0xFFFF0000u);
    } else {
      x[0] = __uint_as_float((uint32_t)*p << 16);
    }
  } else {
    if constexpr (N == 4) { const float4 v = *reinterpret_cast<const float4*>(p); x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w; }
    else if constexpr (N == 2) { const float2 v = *reinterpret_cast<const float2*>(p); x[0] = v.x; x[1] = v.y; }
    else x[0] = *p;
  }
}
// The normalised, scaled and shifted value as the fused LayerNorm + maxout kernels (forward and backward) both
// compute it, rounded to T: the window maxima are decided on exactly these numbers on both sides.
template <typename T>
__device__ __forceinline__ float ln_affine_rounded(float v, float mu, float r, float g, float b) {
  return V8<T>::rounded(__builtin_fmaf((v - mu) * r, g, b));
}

// NIT = chunks per lane held in registers (d <= NIT * 512).
// MAXK = 2, 4, 8: the output is maxout_MAXK of the normalised row (y is then [rows, d / MAXK]; the normalised row
// itself is not stored); MAXK = -1: statistics only.
// DEC: the input row arrives as int8 codes + one fp32 scale per 64 elements (stage-boundary codec); the
// decoded row (code * scale rounded to T, exactly what the stand-alone decode kernel writes) is stored to
// xdec and normalised.
template <typename T, int NIT, bool DEC, int MAXK = 0>
__global__ __launch_bounds__(kLnThreads) void ln_fwd_kernel(const T* __restrict__ x, const T* __restrict__ gamma,
                                                            const T* __restrict__ beta, T* __restrict__ y,
                                                            float* __restrict__ mean, float* __restrict__ rstd,
                                                            int rows, int d, float eps,
                                                            const int8_t* __restrict__ codes,
                                                            const void* __restrict__ scales, T* __restrict__ xdec,
                                                            bool scales16) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int nchunk = d >> 3;
  const float inv_d = 1.0f / (float)d;
  // The row stays in registers as loaded (Raw: 4 registers per 8 bf16 values) and is unpacked once per pass —
  // a third of the registers of an unpacked copy, which is what lets enough wavefronts reside to cover the loads.
  typedef typename V8<T>::Raw Raw;
  for (int row = blockIdx.x * kLnWaves + wave; row < rows; row += gridDim.x * kLnWaves) {
    const T* xr = x + (size_t)row * d;
    Raw raw[NIT];
    float s = 0.f;
    // The loads carry no lane predicate (a chunk index past the row's end is clamped to the last chunk, whose value is
    // then simply not used): a predicated load sits in a branch of its own and is waited for before the next one is
    // issued, eight memory round trips in a row instead of one.
    if constexpr (DEC) {
      uint2 cw[NIT];
      float sc[NIT];
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        const size_t e0 = (size_t)row * d + (size_t)min(lane + it * 64, nchunk - 1) * 8;
        cw[it] = *reinterpret_cast<const uint2*>(codes + e0);
        sc[it] = block_scale_load(scales, e0 >> 6, scales16);
      }
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        const int c = lane + it * 64;
        const uint32_t w[2] = {cw[it].x, cw[it].y};
        float t[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) t[i] = (float)(int)(int8_t)((w[i >> 2] >> (8 * (i & 3))) & 0xFF) * sc[it];
        if (c < nchunk) V8<T>::store(xdec + (size_t)row * d + (size_t)c * 8, t);
        raw[it] = V8<T>::make_raw(t);                                  // the values just stored
      }
    } else {
#pragma unroll
      for (int it = 0; it < NIT; ++it) raw[it] = V8<T>::load_raw(xr + min(lane + it * 64, nchunk - 1) * 8);
    }
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      if (lane + it * 64 < nchunk) {
        float v[8];
        V8<T>::unpack(raw[it], v);
#pragma unroll
        for (int i = 0; i < 8; ++i) s += v[i];
      }
    }
    const float mu = wave_sum(s) * inv_d;
    float q = 0.f;
#pragma unroll
    for (int it = 0; it < NIT; ++it) V8<T>::opaque(raw[it]);
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      if (lane + it * 64 < nchunk) {
        float v[8];
        V8<T>::unpack(raw[it], v);
#pragma unroll
        for (int i = 0; i < 8; ++i) { const float t = v[i] - mu; q += t * t; }
      }
    }
    const float var = wave_sum(q) * inv_d;
    const float r = 1.0f / sqrtf(var + eps);
#pragma unroll
    for (int it = 0; it < NIT; ++it) V8<T>::opaque(raw[it]);
    if constexpr (MAXK == 0) {
      T* yr = y + (size_t)row * d;
      // gamma and beta of all chunks are requested at once, without lane predicates (see the row loads), in two
      // halves so that they do not double the registers of the kernel
      constexpr int HN = NIT > 1 ? NIT / 2 : 1;
#pragma unroll
      for (int h0 = 0; h0 < NIT; h0 += HN) {
        Raw graw[HN], braw[HN];
#pragma unroll
        for (int k = 0; k < HN; ++k) {
          const int cl = min(lane + (h0 + k) * 64, nchunk - 1);
          graw[k] = V8<T>::load_raw(gamma + cl * 8);
          braw[k] = V8<T>::load_raw(beta + cl * 8);
        }
#pragma unroll
        for (int k = 0; k < HN; ++k) {
          const int c = lane + (h0 + k) * 64;
          float v[8], g[8], b[8], o[8];
          V8<T>::unpack(raw[h0 + k], v);
          V8<T>::unpack(graw[k], g);
          V8<T>::unpack(braw[k], b);
#pragma unroll
          for (int i = 0; i < 8; ++i) o[i] = (v[i] - mu) * r * g[i] + b[i];
          if (c < nchunk) V8<T>::store(yr + c * 8, o);
        }
      }
    } else if constexpr (MAXK > 0) {
      T* zr = y + (size_t)row * (d / MAXK);
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        const int c = lane + it * 64;
        if (c < nchunk) {
          float v[8], g[8], b[8], o[8];
          V8<T>::unpack(raw[it], v);
          V8<T>::load(gamma + c * 8, g);
          V8<T>::load(beta + c * 8, b);
#pragma unroll
          for (int w = 0; w < 8 / MAXK; ++w) {
            float m = ln_affine_rounded<T>(v[w * MAXK], mu, r, g[w * MAXK], b[w * MAXK]);
#pragma unroll
            for (int i = 1; i < MAXK; ++i)
              m = fmaxf(m, ln_affine_rounded<T>(v[w * MAXK + i], mu, r, g[w * MAXK + i], b[w * MAXK + i]));
            o[w] = m;
          }
          store_small<T, 8 / MAXK>(zr + c * (8 / MAXK), o);
        }
      }
    }
    if (lane == 0) { mean[row] = mu; rstd[row] = r; }
  }
}

// Backward.  The four wavefronts of a workgroup split the COLUMNS of a row (a quarter each), so a lane
// carries only d/256 dgamma / dbeta partial sums; the two row statistics are combined across the
// wavefronts through LDS, four rows per barrier.  A workgroup walks rpb rows and writes its
// column partials to partial[gridDim.x][2][d] (dgamma then dbeta); a fixed-order second stage adds them up.
// ENC: dx leaves int8-encoded (stage-boundary codec): a lane octet holds one 64-element block of the
// row (needs d % 256 == 0 so that blocks do not straddle wavefronts); the values are rounded to T first,
// so codes and scales equal those of the stand-alone encode kernel on the stored dx.
constexpr int kLnBatch = 4;                  // rows per barrier
// MAXK = 2, 4, 8: dy is the gradient of maxout_MAXK of the normalised row ([rows, d / MAXK]); the normalised row is
// recomputed from x (beta is needed for that) and each window's gradient goes to its first maximum.
template <typename T, int NITQ, bool ENC, int MAXK = 0>
__global__ __launch_bounds__(kLnThreads) void ln_bwd_kernel(const T* __restrict__ dy, const T* __restrict__ x,
                                                            const float* __restrict__ mean,
                                                            const float* __restrict__ rstd,
                                                            const T* __restrict__ gamma, const T* __restrict__ dres,
                                                            T* __restrict__ dx, float* __restrict__ partial, int rows,
                                                            int d, int8_t* __restrict__ codes,
                                                            void* __restrict__ scales, int rpb,
                                                            const T* __restrict__ beta = nullptr,
                                                            bool scales16 = false) {
  __shared__ float red[2][kLnBatch][kLnWaves][2];
  typedef typename V8<T>::Raw Raw;
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int cq = d >> 5;                       // chunks per wavefront (a quarter of d/8)
  const int cbase = wave * cq;
  const float inv_d = 1.0f / (float)d;
  Raw graw[NITQ], braw[MAXK > 0 ? NITQ : 1];
  float pg[NITQ][8], pb[NITQ][8];
#pragma unroll
  for (int it = 0; it < NITQ; ++it) {
    const int c = lane + it * 64;
#pragma unroll
    for (int i = 0; i < 8; ++i) { pg[it][i] = 0.f; pb[it][i] = 0.f; }
    graw[it] = V8<T>::load_raw(gamma + (size_t)(cbase + (c < cq ? c : 0)) * 8);
    if constexpr (MAXK > 0) braw[it] = V8<T>::load_raw(beta + (size_t)(cbase + (c < cq ? c : 0)) * 8);
  }
  const int row0 = blockIdx.x * rpb;
  for (int b0 = 0; b0 < rpb; b0 += kLnBatch) {
    const int par = (b0 / kLnBatch) & 1;
    // The residual gradient is only needed behind the barrier.  Where the registers allow it (four more per chunk
    // and row) it is requested with x and dy and arrives meanwhile; else it is loaded where it is used.
    constexpr bool kEarlyRes = NITQ * sizeof(T) <= 4;
    Raw xraw[kLnBatch][NITQ], dyraw[kLnBatch][NITQ], rraw[kLnBatch][kEarlyRes ? NITQ : 1];
    float mu[kLnBatch], rs[kLnBatch];
    if constexpr (MAXK == 0) {
      // All loads of the batch are issued first and carry no lane predicate (row and chunk indices past the end are
      // clamped, the values then not used): a predicated load sits in a branch of its own and is waited for before
      // the next one is issued, eight memory round trips per batch instead of one.
#pragma unroll
      for (int r = 0; r < kLnBatch; ++r) {
        const size_t rowc = (size_t)min(row0 + b0 + r, rows - 1);
#pragma unroll
        for (int it = 0; it < NITQ; ++it) {
          const size_t e0 = rowc * d + (size_t)(cbase + min(lane + it * 64, cq - 1)) * 8;
          xraw[r][it] = V8<T>::load_raw(x + e0);
          dyraw[r][it] = V8<T>::load_raw(dy + e0);
          if constexpr (kEarlyRes) {
            if (dres) rraw[r][it] = V8<T>::load_raw(dres + e0);
          }
        }
      }
    }
#pragma unroll
    for (int r = 0; r < kLnBatch; ++r) {
      const int row = row0 + b0 + r;
      float s1 = 0.f, s2 = 0.f;
      mu[r] = 0.f; rs[r] = 0.f;
      if (row < rows) {
        mu[r] = mean[row]; rs[r] = rstd[row];
#pragma unroll
        for (int it = 0; it < NITQ; ++it) {
          const int c = lane + it * 64;
          if (c < cq) {
            if constexpr (MAXK > 0) {
              xraw[r][it] = V8<T>::load_raw(x + (size_t)row * d + (size_t)(cbase + c) * 8);
              if constexpr (kEarlyRes) {
                if (dres) rraw[r][it] = V8<T>::load_raw(dres + (size_t)row * d + (size_t)(cbase + c) * 8);
              }
            }
            float xv[8], dv[8], g[8];
            V8<T>::unpack(xraw[r][it], xv);
            V8<T>::unpack(graw[it], g);
            if constexpr (MAXK > 0) {
              float b[8], dz[8];
              V8<T>::unpack(braw[it], b);
              load_small<T, 8 / MAXK>(dy + (size_t)row * (d / MAXK) + (size_t)(cbase + c) * (8 / MAXK), dz);
#pragma unroll
              for (int w = 0; w < 8 / MAXK; ++w) {
                int arg = 0;
                float m = ln_affine_rounded<T>(xv[w * MAXK], mu[r], rs[r], g[w * MAXK], b[w * MAXK]);
#pragma unroll
                for (int i = 1; i < MAXK; ++i) {
                  const float a = ln_affine_rounded<T>(xv[w * MAXK + i], mu[r], rs[r], g[w * MAXK + i], b[w * MAXK + i]);
                  if (a > m) { m = a; arg = i; }      // strict: ties keep the first
                }
#pragma unroll
                for (int i = 0; i < MAXK; ++i) dv[w * MAXK + i] = i == arg ? dz[w] : 0.0f;
              }
              dyraw[r][it] = V8<T>::make_raw(dv);     // exact: dz values and zeros are of type T
            } else {
              V8<T>::unpack(dyraw[r][it], dv);
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) {
              const float xh = (xv[i] - mu[r]) * rs[r];
              const float t = dv[i] * g[i];
              s1 += t;
              s2 += t * xh;
              pg[it][i] += dv[i] * xh;
              pb[it][i] += dv[i];
            }
          }
        }
      }
      s1 = wave_sum(s1);
      s2 = wave_sum(s2);
      if (lane == 0) { red[par][r][wave][0] = s1; red[par][r][wave][1] = s2; }
    }
    __syncthreads();   // the other parity's slots are rewritten only after the next barrier
#pragma unroll
    for (int r = 0; r < kLnBatch; ++r) {
      const int row = row0 + b0 + r;
      if (row >= rows) continue;
      const float m1 = (((red[par][r][0][0] + red[par][r][1][0]) + red[par][r][2][0]) + red[par][r][3][0]) * inv_d;
      const float m2 = (((red[par][r][0][1] + red[par][r][1][1]) + red[par][r][2][1]) + red[par][r][3][1]) * inv_d;
#pragma unroll
      for (int it = 0; it < NITQ; ++it) {
        const int c = lane + it * 64;
        if (c < cq) {
          float res[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}, o[8], xv[8], dv[8], g[8];
          if constexpr (kEarlyRes) {
            if (dres) V8<T>::unpack(rraw[r][it], res);
          } else {
            if (dres) V8<T>::load(dres + (size_t)row * d + (size_t)(cbase + c) * 8, res);
          }
          V8<T>::unpack(xraw[r][it], xv);
          V8<T>::unpack(dyraw[r][it], dv);
          V8<T>::unpack(graw[it], g);
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            // written out operation by operation: the storing and the int8-encoding instantiation must round
            // the same fp32 value, whatever the optimiser would make of an expression
            const float xh = (xv[i] - mu[r]) * rs[r];
            const float t = __builtin_fmaf(-xh, m2, dv[i] * g[i] - m1);
            o[i] = __builtin_fmaf(rs[r], t, res[i]);
          }
          if constexpr (ENC) {
            const size_t e0 = (size_t)row * d + (size_t)(cbase + c) * 8;
            float amax = 0.f;
#pragma unroll
            for (int i = 0; i < 8; ++i) { o[i] = V8<T>::rounded(o[i]); amax = fmaxf(amax, fabsf(o[i])); }
            amax = fmaxf(amax, __shfl_xor(amax, 1, 64));
            amax = fmaxf(amax, __shfl_xor(amax, 2, 64));
            amax = fmaxf(amax, __shfl_xor(amax, 4, 64));
            const float sc = block_scale_rounded(amax / 127.0f, scales16);
            uint32_t w[2] = {0u, 0u};
            if (sc != 0.0f) {
              const BlockDivisor div(sc);
#pragma unroll
              for (int i = 0; i < 8; ++i) {
                const float q = fminf(fmaxf(rintf(div.quotient(o[i])), -127.0f), 127.0f);
                w[i >> 2] |= ((uint32_t)(int)q & 0xFFu) << (8 * (i & 3));
              }
            }
            *reinterpret_cast<uint2*>(codes + e0) = make_uint2(w[0], w[1]);
            if ((lane & 7) == 0) block_scale_store(scales, e0 >> 6, sc, scales16);
          } else {
            V8<T>::store(dx + (size_t)row * d + (size_t)(cbase + c) * 8, o);
          }
        }
      }
    }
  }
  float* out = partial + (size_t)blockIdx.x * 2 * d;
#pragma unroll
  for (int it = 0; it < NITQ; ++it) {
    const int c = lane + it * 64;
    if (c < cq) {
      *reinterpret_cast<float4*>(out + (size_t)(cbase + c) * 8) = make_float4(pg[it][0], pg[it][1], pg[it][2], pg[it][3]);
      *reinterpret_cast<float4*>(out + (size_t)(cbase + c) * 8 + 4) = make_float4(pg[it][4], pg[it][5], pg[it][6], pg[it][7]);
      *reinterpret_cast<float4*>(out + d + (size_t)(cbase + c) * 8) = make_float4(pb[it][0], pb[it][1], pb[it][2], pb[it][3]);
      *reinterpret_cast<float4*>(out + d + (size_t)(cbase + c) * 8 + 4) = make_float4(pb[it][4], pb[it][5], pb[it][6], pb[it][7]);
    }
  }
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
// blockIdx.y = 1 (LayerNorm backward: dbeta next to dgamma in one launch) takes partial + C and out2.
__global__ __launch_bounds__(256) void reduce_rows_accum_kernel(const float* __restrict__ partial, int P, int C,
                                                                size_t stride, float* __restrict__ out,
                                                                float* __restrict__ out2) {
  __shared__ float red[4][64];
  if (blockIdx.y == 1) { partial += C; out = out2; }
  const int c = blockIdx.x * 64 + (threadIdx.x & 63);
  const int rg = threadIdx.x >> 6;
  const int per = (P + 3) / 4;
  const int p0 = rg * per, p1 = min(P, p0 + per);
  float s = 0.f;
  if (c < C) {
    // eight independent running sums (fixed assignment p mod 8, fixed combine order) keep loads in flight
    float a[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    int p = p0;
    for (; p + 8 <= p1; p += 8) {
#pragma unroll
      for (int u = 0; u < 8; ++u) a[u] += partial[(size_t)(p + u) * stride + c];
    }
    for (int u = 0; p < p1; ++p, ++u) a[u] += partial[(size_t)p * stride + c];
    s = ((a[0] + a[1]) + (a[2] + a[3])) + ((a[4] + a[5]) + (a[6] + a[7]));
  }
  red[rg][threadIdx.x & 63] = s;
  __syncthreads();
  if (rg == 0 && c < C) {
    const int l = threadIdx.x & 63;
    out[c] += ((red[0][l] + red[1][l]) + red[2][l]) + red[3][l];
  }
}

template <typename T, bool DEC, int MAXK = 0>
swarm_status ln_fwd_dispatch(const T* x, const T* g, const T* b, T* y, float* mean, float* rstd, int rows, int d,
                             float eps, const int8_t* codes, const void* scales, T* xdec, hipStream_t st,
                             bool scales16 = false) {
  const int grid = std::min((rows + kLnWaves - 1) / kLnWaves, 256 * 8);
#define LN_FWD(NIT)                                                                                           \
  hipLaunchKernelGGL((ln_fwd_kernel<T, NIT, DEC, MAXK>), dim3(grid), dim3(kLnThreads), 0, st, x, g, b, y, mean, \
                     rstd, rows, d, eps, codes, scales, xdec, scales16)
  if (d <= 512) LN_FWD(1);
  else if (d <= 1024) LN_FWD(2);
  else if (d <= 2048) LN_FWD(4);
  else if (d <= 4096) LN_FWD(8);
  else if (d <= 8192) LN_FWD(16);
  else return SWARM_ERR_SHAPE;
#undef LN_FWD
  return launch_status();
}

template <typename T, bool ENC, int MAXK = 0>
swarm_status ln_bwd_dispatch(const T* dy, const T* x, const float* mean, const float* rstd, const T* g,
                             const T* dres, T* dx, float* partial, int rows, int d, int8_t* codes, void* scales,
                             hipStream_t st, const T* beta = nullptr, bool scales16 = false) {
  const int rpb = ln_rows_per_block(rows);
  const int grid = (rows + rpb - 1) / rpb;
#define LN_BWD(NITQ)                                                                                                \
  hipLaunchKernelGGL((ln_bwd_kernel<T, NITQ, ENC, MAXK>), dim3(grid), dim3(kLnThreads), 0, st, dy, x, mean, rstd, g, \
                     dres, dx, partial, rows, d, codes, scales, rpb, beta, scales16)
  if (d <= 2048) LN_BWD(1);
  else if (d <= 4096) LN_BWD(2);
  else if (d <= 8192) LN_BWD(4);
  else return SWARM_ERR_SHAPE;
#undef LN_BWD
  return launch_status();
}

}  // namespace

swarm_status layernorm_fwd(const void* x, const void* gamma, const void* beta, void* y, float* mean, float* rstd,
                           int T, int d, float eps, bool bf16, hipStream_t st) {
  if (bf16)
    return ln_fwd_dispatch<bf16_raw, false>((const bf16_raw*)x, (const bf16_raw*)gamma, (const bf16_raw*)beta,
                                            (bf16_raw*)y, mean, rstd, T, d, eps, nullptr, nullptr, nullptr, st);
  return ln_fwd_dispatch<float, false>((const float*)x, (const float*)gamma, (const float*)beta, (float*)y, mean,
                                       rstd, T, d, eps, nullptr, nullptr, nullptr, st);
}

swarm_status layernorm_fwd_decode(const int8_t* codes, const void* scales, void* xdec, const void* gamma,
                                  const void* beta, void* y, float* mean, float* rstd, int T, int d, float eps,
                                  bool bf16, hipStream_t st, bool scales16) {
  if (!bf16) return SWARM_ERR_SHAPE;     // the stage fuses the codec for bf16 activations only
  return ln_fwd_dispatch<bf16_raw, true>(nullptr, (const bf16_raw*)gamma, (const bf16_raw*)beta, (bf16_raw*)y, mean,
                                         rstd, T, d, eps, codes, scales, (bf16_raw*)xdec, st, scales16);
}

size_t layernorm_bwd_scratch_floats(int T, int d) {
  const int rpb = ln_rows_per_block(T);
  return (size_t)((T + rpb - 1) / rpb) * 2 * d;
}

// codes != nullptr: dx is not written; its int8 encoding goes to codes / scales (needs d % 256 == 0)
swarm_status layernorm_bwd(const void* dy, const void* x, const float* mean, const float* rstd, const void* gamma,
                           const void* dres, void* dx, float* dgamma, float* dbeta, float* partial, int T, int d,
                           bool bf16, hipStream_t st, int8_t* codes, void* scales, bool scales16) {
  swarm_status s;
  if (codes && (d % 256 || !bf16)) return SWARM_ERR_SHAPE;     // the stage fuses the codec for bf16 activations only
  if (bf16) {
    const bf16_raw *a = (const bf16_raw*)dy, *b = (const bf16_raw*)x, *g = (const bf16_raw*)gamma,
                   *r = (const bf16_raw*)dres;
    s = codes ? ln_bwd_dispatch<bf16_raw, true>(a, b, mean, rstd, g, r, nullptr, partial, T, d, codes, scales, st,
                                                nullptr, scales16)
              : ln_bwd_dispatch<bf16_raw, false>(a, b, mean, rstd, g, r, (bf16_raw*)dx, partial, T, d, nullptr, nullptr,
                                                 st);
  } else {
    const float *a = (const float*)dy, *b = (const float*)x, *g = (const float*)gamma, *r = (const float*)dres;
    s = ln_bwd_dispatch<float, false>(a, b, mean, rstd, g, r, (float*)dx, partial, T, d, nullptr, nullptr, st);
  }
  if (s != SWARM_OK) return s;
  const int P = (T + ln_rows_per_block(T) - 1) / ln_rows_per_block(T);
  const int grid = (d + 63) / 64;
  hipLaunchKernelGGL(reduce_rows_accum_kernel, dim3(grid, 2), dim3(256), 0, st, partial, P, d, (size_t)2 * d, dgamma,
                     dbeta);
  return launch_status();
}

// Fused LayerNorm + maxout_k (k in {2, 4, 8}, d % 8 == 0; anything else: SWARM_ERR_SHAPE, nothing launched).
// k = -1: mean and rstd only.
swarm_status layernorm_fwd_maxout(const void* x, const void* gamma, const void* beta, void* z, float* mean, float* rstd,
                                  int T, int d, int k, float eps, bool bf16, hipStream_t st) {
#define LN_MO(TT, K)                                                                                               \
  return ln_fwd_dispatch<TT, false, K>((const TT*)x, (const TT*)gamma, (const TT*)beta, (TT*)z, mean, rstd, T, d, eps, \
                                       nullptr, nullptr, nullptr, st)
  if (bf16) {
    if (k == 2) LN_MO(bf16_raw, 2);
    if (k == 4) LN_MO(bf16_raw, 4);
    if (k == 8) LN_MO(bf16_raw, 8);
    if (k == -1) LN_MO(bf16_raw, -1);
  } else {
    if (k == 2) LN_MO(float, 2);
    if (k == 4) LN_MO(float, 4);
    if (k == 8) LN_MO(float, 8);
    if (k == -1) LN_MO(float, -1);
  }
#undef LN_MO
  return SWARM_ERR_SHAPE;
}

// dx = LN-backward of the gradient that maxout_k routes from dz [T, d / k] to the first maximum of every window of
// the normalised row (recomputed from x, mean, rstd); dgamma, dbeta += as in layernorm_bwd.
swarm_status layernorm_bwd_maxout(const void* dz, const void* x, const float* mean, const float* rstd,
                                  const void* gamma, const void* beta, void* dx, float* dgamma, float* dbeta,
                                  float* partial, int T, int d, int k, bool bf16, hipStream_t st) {
  swarm_status s = SWARM_ERR_SHAPE;
#define LN_MOB(TT, K)                                                                                             \
  s = ln_bwd_dispatch<TT, false, K>((const TT*)dz, (const TT*)x, mean, rstd, (const TT*)gamma, (const TT*)nullptr, \
                                    (TT*)dx, partial, T, d, nullptr, nullptr, st, (const TT*)beta)
  if (bf16) {
    if (k == 2) LN_MOB(bf16_raw, 2);
    else if (k == 4) LN_MOB(bf16_raw, 4);
    else if (k == 8) LN_MOB(bf16_raw, 8);
  } else {
    if (k == 2) LN_MOB(float, 2);
    else if (k == 4) LN_MOB(float, 4);
    else if (k == 8) LN_MOB(float, 8);
  }
#undef LN_MOB
  if (s != SWARM_OK) return s;
  const int P = (T + ln_rows_per_block(T) - 1) / ln_rows_per_block(T);
  hipLaunchKernelGGL(reduce_rows_accum_kernel, dim3((d + 63) / 64, 2), dim3(256), 0, st, partial, P, d, (size_t)2 * d,
                     dgamma, dbeta);
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
                     out, (float*)nullptr);
  return launch_status();
}

}  // namespace swarm
