// Micro-benchmarks behind the roofline discussion of the bf16 GEMM.  Instrumented build only (libswarm_hooks.so);
// nothing here is on the stage path.
//   mfma_rate : a loop of nothing but MFMAs on register operands, in the GEMM kernel's own shape (8 wavefronts per
//               workgroup, 128 accumulator registers per lane, 32 / 8 independent MFMAs per iteration) - the rate the
//               matrix pipes sustain when nothing else runs, for constant or random operand bits;
//   lds_read  : a loop of nothing but LDS fragment reads with the GEMM kernel's two read shapes and swizzles.
// Each workgroup also records the 100 MHz wall clock and the shader clock counter at its start and end, which gives
// the clock the chip ran at under that load.
#include "gemm_bf16_common.h"

namespace swarm {
namespace {

// [0] wall clock at start, [1] at end, [2] shader-cycle counter at start, [3] at end
__device__ __forceinline__ void stamp_clocks(long long* out, bool end) {
  if (threadIdx.x == 0) {
    out[(size_t)blockIdx.x * 4 + (end ? 1 : 0)] = wall_clock64();
    out[(size_t)blockIdx.x * 4 + (end ? 3 : 2)] = clock64();
  }
}

template <int SHAPE>   // 0: v_mfma_f32_16x16x32_bf16, 1: v_mfma_f32_32x32x16_bf16
__global__ __launch_bounds__(512) void mfma_rate_kernel(const uint4* __restrict__ operands, float* __restrict__ sink,
                                                        int iters, long long* __restrict__ clocks) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  constexpr int NA = SHAPE == 0 ? 8 : 4, NB = SHAPE == 0 ? 4 : 2;
  bf16x8 a[NA], b[NB];
  // 12 (6) fragments per wavefront, different bits per wavefront and lane
#pragma unroll
  for (int i = 0; i < NA; ++i) a[i] = __builtin_bit_cast(bf16x8, operands[((wave * 12 + i) * 64 + lane)]);
#pragma unroll
  for (int j = 0; j < NB; ++j) b[j] = __builtin_bit_cast(bf16x8, operands[((wave * 12 + 8 + j) * 64 + lane)]);
  stamp_clocks(clocks, false);
  float total = 0.f;
  if constexpr (SHAPE == 0) {
    f32x4 acc[NA][NB];
#pragma unroll
    for (int i = 0; i < NA; ++i)
#pragma unroll
      for (int j = 0; j < NB; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int i = 0; i < NA; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < NA; ++i)
#pragma unroll
      for (int j = 0; j < NB; ++j) total += acc[i][j][0] + acc[i][j][1] + acc[i][j][2] + acc[i][j][3];
  } else {
    f32x16 acc[NA][NB];
#pragma unroll
    for (int i = 0; i < NA; ++i)
#pragma unroll
      for (int j = 0; j < NB; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int i = 0; i < NA; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < NA; ++i)
#pragma unroll
      for (int j = 0; j < NB; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) total += acc[i][j][r];
  }
  stamp_clocks(clocks, true);
  sink[(size_t)blockIdx.x * 512 + threadIdx.x] = total;
}

// 64 KiB of LDS (one operand stage of the 256 x 256 kernel), read-only loop.  TR = false: ds_read_b128 fragments of
// a [rows][64 k] tile with the 16 x 16 x 32 kernel's chunk swizzle; TR = true: ds_read_b64_tr_b16 pairs from a
// [k][256] tile with its swizzle.  12 fragments per iteration and wavefront, as a sub-step of the GEMM reads them.
template <bool TR>
__global__ __launch_bounds__(512) void lds_read_kernel(float* __restrict__ sink, int iters,
                                                       long long* __restrict__ clocks) {
  extern __shared__ __attribute__((aligned(1024))) bf16_raw lds[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int i = threadIdx.x; i < 32768; i += 512) lds[i] = (bf16_raw)(i * 2654435761u >> 16);
  __syncthreads();
  const int wm = wave >> 2, wn = wave & 3;
  const int l16 = lane & 15, q = lane >> 4;
  uint32_t x0 = 0, x1 = 0, x2 = 0, x3 = 0;
  stamp_clocks(clocks, false);
  for (int it = 0; it < iters; ++it) {
    const int kk = it & 1;
    u32x4_t v[12];   // all twelve requests are in flight before the one wait, as in the GEMM's sub-step
#pragma unroll
    for (int f = 0; f < 12; ++f) {
      // fragments 0..7: the wavefront's A rows (tile rows 0..255), 8..11: its B columns (rows 256..511 of the stage)
      const int row_base = f < 8 ? wm * 128 + 16 * f : 256 + wn * 64 + 16 * (f - 8);
      if constexpr (!TR) {
        const int row = row_base + l16;
        const int chunk = (4 * kk + q) ^ (l16 & 7);
        const uint32_t addr =
            (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)(lds + row * 64 + chunk * 8);
        asm volatile("ds_read_b128 %0, %1" : "=v"(v[f]) : "v"(addr) : "memory");
      } else {
        // [64 k][256 columns] per operand; the stage holds A then B (2 x 32 KiB)
        const int col = (row_base & 255) + 4 * (l16 & 3);
        const int kq = l16 >> 2;
        const int chunk = (col >> 3) ^ (4 * kq) ^ (2 * (q & 1));
        const int krow = 32 * kk + 8 * q + kq;
        const bf16_raw* p0 = lds + (row_base >> 8) * 16384 + krow * 256 + chunk * 8 + (col & 4);
        const uint32_t addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p0;
        uint2 lo, hi;
        asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(lo) : "v"(addr) : "memory");
        asm volatile("ds_read_b64_tr_b16 %0, %1 offset:2048" : "=v"(hi) : "v"(addr) : "memory");
        v[f] = u32x4_t{lo.x, lo.y, hi.x, hi.y};
      }
    }
    __builtin_amdgcn_s_waitcnt(0xC07F);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int f = 0; f < 12; ++f) { x0 ^= v[f][0]; x1 ^= v[f][1]; x2 ^= v[f][2]; x3 ^= v[f][3]; }
  }
  stamp_clocks(clocks, true);
  sink[(size_t)blockIdx.x * 512 + threadIdx.x] = __uint_as_float((x0 ^ x1 ^ x2 ^ x3) & 0x3FFFFFFFu);
}

// Vector-arithmetic rate of ONE workgroup per compute unit (96 KiB of LDS requested, so no second one fits) of
// THREADS / 64 wavefronts: every lane runs `iters` rounds of the GEMM epilogue's GeLU on 8 independent values.
// 256 threads = one wavefront per SIMD, 512 = two.
template <int THREADS>
__global__ __launch_bounds__(THREADS) void valu_rate_kernel(const float* __restrict__ in, float* __restrict__ sink,
                                                             int iters, long long* __restrict__ clocks) {
  float x[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) x[e] = in[(threadIdx.x * 8 + e) & 4095];
  stamp_clocks(clocks, false);
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] = gelu_fast(x[e]) + 0.25f;
  }
  stamp_clocks(clocks, true);
  float t = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) t += x[e];
  sink[(size_t)blockIdx.x * THREADS + threadIdx.x] = t;
}

}  // namespace
}  // namespace swarm

using namespace swarm;

// in: 4096 floats; sink: workgroups x 512 floats; clocks: workgroups x 4 int64.  waves_per_simd: 1 or 2.
extern "C" int swarm_microbench_valu_rate(int waves_per_simd, const float* in, float* sink, long long* clocks, int iters,
                                          int workgroups, void* stream) {
  if (!in || !sink || !clocks || iters < 1 || workgroups < 1 || (waves_per_simd != 1 && waves_per_simd != 2))
    return SWARM_ERR_SHAPE;
  static LdsOptIn opted[2];
  const void* k = waves_per_simd == 1 ? (const void*)valu_rate_kernel<256> : (const void*)valu_rate_kernel<512>;
  if (lds_opt_in(k, 98304, opted[waves_per_simd - 1]) != SWARM_OK) return SWARM_ERR_LAUNCH;
  if (waves_per_simd == 1)
    hipLaunchKernelGGL(valu_rate_kernel<256>, dim3(workgroups), dim3(256), 98304, (hipStream_t)stream, in, sink, iters, clocks);
  else
    hipLaunchKernelGGL(valu_rate_kernel<512>, dim3(workgroups), dim3(512), 98304, (hipStream_t)stream, in, sink, iters, clocks);
  return launch_status();
}

// operands: 8 x 12 x 64 uint4 (device); sink: workgroups x 512 floats; clocks: workgroups x 4 int64.
// Launches the loop once on `stream`; the caller times it.  shape 0: 16 x 16 x 32 (32 MFMAs per iteration and
// wavefront, 16384 flops each), 1: 32 x 32 x 16 (8 MFMAs per iteration, 32768 flops each).
extern "C" int swarm_microbench_mfma_rate(int shape, const void* operands, float* sink, long long* clocks, int iters,
                                          int workgroups, void* stream) {
  if (!operands || !sink || !clocks || iters < 1 || workgroups < 1 || (shape != 0 && shape != 1)) return SWARM_ERR_SHAPE;
  if (shape == 0)
    hipLaunchKernelGGL(mfma_rate_kernel<0>, dim3(workgroups), dim3(512), 0, (hipStream_t)stream,
                       (const uint4*)operands, sink, iters, clocks);
  else
    hipLaunchKernelGGL(mfma_rate_kernel<1>, dim3(workgroups), dim3(512), 0, (hipStream_t)stream,
                       (const uint4*)operands, sink, iters, clocks);
  return launch_status();
}

// transposed = 0: ds_read_b128 (1 KiB per wavefront instruction), 1: ds_read_b64_tr_b16 pairs (2 x 512 B).
// 12 fragments of 1 KiB per iteration and wavefront either way.
extern "C" int swarm_microbench_lds_read(int transposed, float* sink, long long* clocks, int iters, int workgroups,
                                         void* stream) {
  if (!sink || !clocks || iters < 1 || workgroups < 1) return SWARM_ERR_SHAPE;
  static LdsOptIn opted[2];
  const void* k = transposed ? (const void*)lds_read_kernel<true> : (const void*)lds_read_kernel<false>;
  if (lds_opt_in(k, 65536, opted[transposed ? 1 : 0]) != SWARM_OK) return SWARM_ERR_LAUNCH;
  if (transposed)
    hipLaunchKernelGGL(lds_read_kernel<true>, dim3(workgroups), dim3(512), 65536, (hipStream_t)stream, sink, iters, clocks);
  else
    hipLaunchKernelGGL(lds_read_kernel<false>, dim3(workgroups), dim3(512), 65536, (hipStream_t)stream, sink, iters, clocks);
  return launch_status();
}
