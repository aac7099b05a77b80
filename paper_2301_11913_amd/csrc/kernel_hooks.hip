// Kernel-level entry points for unit tests and micro-benchmarks of single kernels.
// They are not part of the stage ABI (include/swarm_stage.h); arguments are device pointers.
#include "kernels.h"

using namespace swarm;

// C[M,N] (+)= A(m,k) B(n,k); layouts and epilogues as in GemmArgs.  dtype: 0 fp32, 1 bf16.
extern "C" int swarm_kernel_gemm(int dtype, int M, int N, int K, const void* A, int lda, int a_trans, const void* B,
                                 int ldb, int b_trans, void* C, int ldc, int epilogue, const void* bias,
                                 const void* aux, int ldaux, void* C2, int ldc2, void* stream) {
  GemmArgs g{};
  g.M = M; g.N = N; g.K = K; g.A = A; g.lda = lda; g.a_trans = a_trans != 0; g.B = B; g.ldb = ldb;
  g.b_trans = b_trans != 0; g.C = C; g.ldc = ldc; g.epilogue = epilogue; g.bias = bias; g.aux = aux;
  g.ldaux = ldaux; g.C2 = C2; g.ldc2 = ldc2;
  return dtype ? gemm_bf16(g, (hipStream_t)stream) : gemm_f32(g, (hipStream_t)stream);
}

// The same with split-K scratch (floats) that the bf16 kernel may use; swarm_kernel_gemm_splitk_floats says how much.
extern "C" size_t swarm_kernel_gemm_splitk_floats(int M, int N) { return gemm_splitk_floats(M, N); }
extern "C" int swarm_kernel_gemm_ws(int M, int N, int K, const void* A, int lda, int a_trans, const void* B, int ldb,
                                    int b_trans, void* C, int ldc, int epilogue, const void* bias, const void* aux,
                                    int ldaux, float* scales, float* splitk_ws, size_t splitk_floats, void* stream) {
  GemmArgs g{};
  g.M = M; g.N = N; g.K = K; g.A = A; g.lda = lda; g.a_trans = a_trans != 0; g.B = B; g.ldb = ldb;
  g.b_trans = b_trans != 0; g.C = C; g.ldc = ldc; g.epilogue = epilogue; g.bias = bias; g.aux = aux;
  g.ldaux = ldaux; g.scales = scales; g.splitk_ws = splitk_ws; g.splitk_floats = splitk_floats;
  return gemm_bf16(g, (hipStream_t)stream);
}

// The same again with phase stamps of the 256 x 256 kernel: stamps [workgroups x 16] int64 (device) receive, per
// workgroup, the 100 MHz wall clock at its start, at the first barrier, behind the loop and when the epilogue's
// stores have left, then the HW_ID and XCC_ID registers, the tile coordinates and the shader cycles spent in the loop.
extern "C" int swarm_kernel_gemm_stamped(int M, int N, int K, const void* A, int lda, int a_trans, const void* B,
                                         int ldb, int b_trans, void* C, int ldc, int epilogue, const void* bias,
                                         const void* aux, int ldaux, long long* stamps, void* stream) {
  GemmArgs g{};
  g.M = M; g.N = N; g.K = K; g.A = A; g.lda = lda; g.a_trans = a_trans != 0; g.B = B; g.ldb = ldb;
  g.b_trans = b_trans != 0; g.C = C; g.ldc = ldc; g.epilogue = epilogue; g.bias = bias; g.aux = aux;
  g.ldaux = ldaux; g.stamps = stamps;
  if (M % 256 || N % 256 || (long)(M / 256) * (N / 256) < 160) return SWARM_ERR_SHAPE;   // one 256 x 256 launch only
  return gemm_bf16(g, (hipStream_t)stream);
}

extern "C" int swarm_kernel_attention_fwd(int dtype, const void* qkv, void* o, float* lse, int B, int S, int H,
                                          int dh, void* stream) {
  return attention_fwd(qkv, o, lse, B, S, H, dh, dtype != 0, (hipStream_t)stream);
}

extern "C" int swarm_kernel_attention_bwd(int dtype, const void* qkv, const void* o, const void* dout,
                                          const float* lse, float* delta, void* dqkv, int B, int S, int H, int dh,
                                          void* stream) {
  return attention_bwd(qkv, o, dout, lse, delta, dqkv, B, S, H, dh, dtype != 0, (hipStream_t)stream);
}

// codes[i] = clamp(rint(x[i] / scale[i]), -127, 127) through BlockDivisor, the shared-reciprocal form of the
// correctly rounded division that the codec kernels use (scale[i] > 0, finite).
namespace {
__global__ __launch_bounds__(256) void quantise_pairs_kernel(const float* __restrict__ x,
                                                             const float* __restrict__ scale, size_t n,
                                                             int8_t* __restrict__ codes) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const BlockDivisor div(scale[i]);
  codes[i] = (int8_t)(int)fminf(fmaxf(rintf(div.quotient(x[i])), -127.0f), 127.0f);
}
}  // namespace
extern "C" int swarm_kernel_quantise_pairs(const float* x, const float* scale, size_t n, int8_t* codes,
                                           void* stream) {
  if (n == 0) return SWARM_OK;
  if (!x || !scale || !codes) return SWARM_ERR_NULL;
  hipLaunchKernelGGL(quantise_pairs_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream, x,
                     scale, n, codes);
  return launch_status();
}
