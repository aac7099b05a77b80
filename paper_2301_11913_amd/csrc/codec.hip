// Blockwise absmax int8 codec for stage-boundary tensors (paper appendix
// "Compression-Aware Architectures", paragraph "Quantized activations").
//
// Bit-exactness contract: every arithmetic step is one IEEE fp32 operation
// (this file is compiled with -ffp-contract=off and without fast-math, so `/`
// is the correctly rounded division and rintf is round-half-to-even).
//
// Layout: one lane owns 8 consecutive elements, so the 8 lanes of an aligned
// lane-octet own one 64-element block; the block absmax is a 3-step xor
// butterfly inside the octet.  A wavefront covers 512 contiguous elements:
// loads are 16 B (bf16) or 2 x 16 B (fp32) per lane, code stores 8 B per lane,
// all fully coalesced.  HBM-bound: 3.0625 B/element from bf16, 5.0625 from fp32.
#include "kernels.h"

namespace swarm {

constexpr int kBlock = 64;        // codec block (elements)
constexpr int kPerLane = 8;       // elements per lane
constexpr int kThreads = 256;

template <typename T> struct Vec8;
template <> struct Vec8<bf16_raw> {
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
template <> struct Vec8<float> {
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

// Block scale as stored: fp32, or its bf16 rounding as a 16-bit pattern (the codes then divide by the ROUNDED scale).
template <typename S> struct ScaleIO;
template <> struct ScaleIO<float> {
  static __device__ __forceinline__ float round(float s) { return s; }
  static __device__ __forceinline__ void store(float* p, float s) { *p = s; }
  static __device__ __forceinline__ float load(const float* p) { return *p; }
};
template <> struct ScaleIO<uint16_t> {
  static __device__ __forceinline__ float round(float s) { return __uint_as_float(float_to_bf16_bits(s) << 16); }
  static __device__ __forceinline__ void store(uint16_t* p, float s) { *p = (uint16_t)(__float_as_uint(s) >> 16); }
  static __device__ __forceinline__ float load(const uint16_t* p) { return __uint_as_float((uint32_t)*p << 16); }
};

__device__ __forceinline__ int quantise(float x, const BlockDivisor& scale) {
  float q = rintf(scale.quotient(x));
  q = fminf(fmaxf(q, -127.0f), 127.0f);
  return (int)q;
}

// Full 8-element groups: n8 = n_elems / 8 groups, each handled by one lane.
template <typename T, typename S = float>
__global__ __launch_bounds__(kThreads) void codec_encode_kernel(const T* __restrict__ src, size_t n_elems,
                                                                int8_t* __restrict__ codes,
                                                                S* __restrict__ scales) {
  const size_t n_groups = (n_elems + kPerLane - 1) / kPerLane;
  const size_t stride = (size_t)gridDim.x * kThreads;
  // all lanes of an octet run the same number of iterations: n_groups is padded to a multiple of 8 below
  const size_t n_groups_pad = (n_groups + 7) & ~(size_t)7;
  for (size_t g = (size_t)blockIdx.x * kThreads + threadIdx.x; g < n_groups_pad; g += stride) {
    const size_t base = g * kPerLane;
    float x[8];
    if (base + kPerLane <= n_elems) {
      Vec8<T>::load(src + base, x);
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) x[i] = (base + i < n_elems) ? Elem<T>::load(src + base + i) : 0.0f;
    }
    float a = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i) a = fmaxf(a, fabsf(x[i]));
    a = fmaxf(a, __shfl_xor(a, 1, 64));
    a = fmaxf(a, __shfl_xor(a, 2, 64));
    a = fmaxf(a, __shfl_xor(a, 4, 64));
    const float scale = ScaleIO<S>::round(a / 127.0f);
    int c[8];
    if (scale == 0.0f) {
#pragma unroll
      for (int i = 0; i < 8; ++i) c[i] = 0;
    } else {
      const BlockDivisor div(scale);
#pragma unroll
      for (int i = 0; i < 8; ++i) c[i] = quantise(x[i], div);
    }
    if (base + kPerLane <= n_elems) {
      uint2 out;
      out.x = (uint32_t)(c[0] & 0xFF) | ((uint32_t)(c[1] & 0xFF) << 8) | ((uint32_t)(c[2] & 0xFF) << 16) |
              ((uint32_t)(c[3] & 0xFF) << 24);
      out.y = (uint32_t)(c[4] & 0xFF) | ((uint32_t)(c[5] & 0xFF) << 8) | ((uint32_t)(c[6] & 0xFF) << 16) |
              ((uint32_t)(c[7] & 0xFF) << 24);
      *reinterpret_cast<uint2*>(codes + base) = out;
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i)
        if (base + i < n_elems) codes[base + i] = (int8_t)c[i];
    }
    if ((g & 7) == 0 && base < n_elems) ScaleIO<S>::store(scales + (g >> 3), scale);
  }
}

template <typename T, typename S = float>
__global__ __launch_bounds__(kThreads) void codec_decode_kernel(const int8_t* __restrict__ codes,
                                                                const S* __restrict__ scales, size_t n_elems,
                                                                T* __restrict__ dst) {
  const size_t n_groups = (n_elems + kPerLane - 1) / kPerLane;
  const size_t stride = (size_t)gridDim.x * kThreads;
  for (size_t g = (size_t)blockIdx.x * kThreads + threadIdx.x; g < n_groups; g += stride) {
    const size_t base = g * kPerLane;
    const float scale = ScaleIO<S>::load(scales + (g >> 3));
    float y[8];
    if (base + kPerLane <= n_elems) {
      uint2 v = *reinterpret_cast<const uint2*>(codes + base);
      uint32_t w[2] = {v.x, v.y};
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        int c = (int)(int8_t)((w[i >> 2] >> (8 * (i & 3))) & 0xFF);
        y[i] = (float)c * scale;
      }
      Vec8<T>::store(dst + base, y);
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i)
        if (base + i < n_elems) Elem<T>::store(dst + base + i, (float)codes[base + i] * scale);
    }
  }
}

static int codec_grid(size_t n_elems) {
  size_t groups = (n_elems + kPerLane - 1) / kPerLane;
  size_t blocks = (groups + kThreads - 1) / kThreads;
  const size_t cap = 256 * 16;   // 16 workgroups per CU, grid-stride beyond that
  return (int)(blocks < cap ? (blocks ? blocks : 1) : cap);
}

swarm_status codec_encode_launch(const void* tensor, size_t n, int8_t* codes, void* scales, bool bf16,
                                 hipStream_t st, bool scales16) {
  if (n == 0) return SWARM_OK;
  const int grid = codec_grid(n);
  const dim3 g(grid), b(kThreads);
  if (bf16 && !scales16)
    hipLaunchKernelGGL((codec_encode_kernel<bf16_raw, float>), g, b, 0, st, (const bf16_raw*)tensor, n, codes, (float*)scales);
  else if (bf16)
    hipLaunchKernelGGL((codec_encode_kernel<bf16_raw, uint16_t>), g, b, 0, st, (const bf16_raw*)tensor, n, codes, (uint16_t*)scales);
  else if (!scales16)
    hipLaunchKernelGGL((codec_encode_kernel<float, float>), g, b, 0, st, (const float*)tensor, n, codes, (float*)scales);
  else
    hipLaunchKernelGGL((codec_encode_kernel<float, uint16_t>), g, b, 0, st, (const float*)tensor, n, codes, (uint16_t*)scales);
  return launch_status();
}

swarm_status codec_decode_launch(const int8_t* codes, const void* scales, size_t n, void* tensor, bool bf16,
                                 hipStream_t st, bool scales16) {
  if (n == 0) return SWARM_OK;
  const int grid = codec_grid(n);
  const dim3 g(grid), b(kThreads);
  if (bf16 && !scales16)
    hipLaunchKernelGGL((codec_decode_kernel<bf16_raw, float>), g, b, 0, st, codes, (const float*)scales, n, (bf16_raw*)tensor);
  else if (bf16)
    hipLaunchKernelGGL((codec_decode_kernel<bf16_raw, uint16_t>), g, b, 0, st, codes, (const uint16_t*)scales, n, (bf16_raw*)tensor);
  else if (!scales16)
    hipLaunchKernelGGL((codec_decode_kernel<float, float>), g, b, 0, st, codes, (const float*)scales, n, (float*)tensor);
  else
    hipLaunchKernelGGL((codec_decode_kernel<float, uint16_t>), g, b, 0, st, codes, (const uint16_t*)scales, n, (float*)tensor);
  return launch_status();
}

}  // namespace swarm

using namespace swarm;

extern "C" swarm_status swarm_codec_encode(const void* tensor, int32_t dtype, size_t n_elems, int32_t block,
                                           int8_t* codes, float* scales, void* hip_stream) {
  if (block != kBlock) return SWARM_ERR_SHAPE;
  if (dtype != SWARM_F32 && dtype != SWARM_BF16) return SWARM_ERR_DTYPE;
  if (n_elems == 0) return SWARM_OK;
  if (!tensor || !codes || !scales) return SWARM_ERR_NULL;
  if (((uintptr_t)tensor & 15) || ((uintptr_t)codes & 7) || ((uintptr_t)scales & 3)) return SWARM_ERR_SHAPE;
  return codec_encode_launch(tensor, n_elems, codes, scales, dtype == SWARM_BF16, (hipStream_t)hip_stream);
}

extern "C" swarm_status swarm_codec_decode(const int8_t* codes, const float* scales, size_t n_elems, int32_t block,
                                           void* tensor, int32_t dtype, void* hip_stream) {
  if (block != kBlock) return SWARM_ERR_SHAPE;
  if (dtype != SWARM_F32 && dtype != SWARM_BF16) return SWARM_ERR_DTYPE;
  if (n_elems == 0) return SWARM_OK;
  if (!tensor || !codes || !scales) return SWARM_ERR_NULL;
  if (((uintptr_t)tensor & 15) || ((uintptr_t)codes & 7) || ((uintptr_t)scales & 3)) return SWARM_ERR_SHAPE;
  return codec_decode_launch(codes, scales, n_elems, tensor, dtype == SWARM_BF16, (hipStream_t)hip_stream);
}

extern "C" swarm_status swarm_codec_encode_s16(const void* tensor, int32_t dtype, size_t n_elems, int32_t block,
                                               int8_t* codes, uint16_t* scales, void* hip_stream) {
  if (block != kBlock) return SWARM_ERR_SHAPE;
  if (dtype != SWARM_F32 && dtype != SWARM_BF16) return SWARM_ERR_DTYPE;
  if (n_elems == 0) return SWARM_OK;
  if (!tensor || !codes || !scales) return SWARM_ERR_NULL;
  if (((uintptr_t)tensor & 15) || ((uintptr_t)codes & 7) || ((uintptr_t)scales & 1)) return SWARM_ERR_SHAPE;
  return codec_encode_launch(tensor, n_elems, codes, scales, dtype == SWARM_BF16, (hipStream_t)hip_stream, true);
}

extern "C" swarm_status swarm_codec_decode_s16(const int8_t* codes, const uint16_t* scales, size_t n_elems,
                                               int32_t block, void* tensor, int32_t dtype, void* hip_stream) {
  if (block != kBlock) return SWARM_ERR_SHAPE;
  if (dtype != SWARM_F32 && dtype != SWARM_BF16) return SWARM_ERR_DTYPE;
  if (n_elems == 0) return SWARM_OK;
  if (!tensor || !codes || !scales) return SWARM_ERR_NULL;
  if (((uintptr_t)tensor & 15) || ((uintptr_t)codes & 7) || ((uintptr_t)scales & 1)) return SWARM_ERR_SHAPE;
  return codec_decode_launch(codes, scales, n_elems, tensor, dtype == SWARM_BF16, (hipStream_t)hip_stream, true);
}
