// Internal launch interface between the stage driver and the kernel files.
// Everything here works on device pointers and enqueues on the given stream.
#pragma once
#include "common.h"

namespace swarm {

// ------------------------------------------------------------------ GEMM
// C[M,N] (+)= sum_k A(m,k) * B(n,k) with fp32 accumulation.
//   a_trans = false: A stored [M,K] (k contiguous, row pitch lda); true: stored [K,M].
//   b_trans = false: B stored [N,K] (k contiguous, row pitch ldb); true: stored [K,N].
// The three uses: forward  y = x W^T      (A = x [T,in],   B = W [out,in]:            F,F)
//                 dgrad    dx = dy W      (A = dy [T,out], B = W [out,in] as [K,N]:    F,T)
//                 wgrad    dW += dy^T x   (A = dy [T,out] as [K,M], B = x [T,in]:      T,T)
enum GemmEpilogue {
  EPI_STORE = 0,       // C = acc                                   (C in the activation dtype)
  EPI_BIAS = 1,        // C = acc + bias[n]
  EPI_BIAS_RESID = 2,  // C = acc + bias[n] + aux[m,n]
  EPI_BIAS_GELU = 3,   // u = acc + bias[n]; C = gelu(u); C2 = u when C2 != nullptr
  EPI_DGELU = 4,       // C = acc * gelu'(aux[m,n])
  EPI_ACCUM_F32 = 5,   // C (fp32) += acc
  EPI_BIAS_RESID_ENCODE = 6,  // x = acc + bias[n] + aux[m,n] rounded to bf16, stored int8-encoded: C = codes, scales
  // The three below exist in the bf16 MFMA kernels only; gemm_bf16 returns SWARM_ERR_SHAPE (nothing launched)
  // for a problem they cannot take, and the caller then uses the unfused kernels.
  EPI_BIAS_ROPE = 7,          // C = acc + bias[n], columns n < rope_cols rotated pairwise (rotary embedding)
  EPI_DGEGLU = 8,             // aux = u [M, 2*split]: C[m,n] = acc * u[m,split+n] * gelu'(u[m,n]),
                              //                       C[m,split+n] = acc * gelu(u[m,n])        (N = split)
  EPI_BIAS_GEGLU = 9          // B = W1 [2*split, K], N = 2*split: u = acc + bias over gate|up,
                              // C[m,j] = gelu(u[m,j]) * u[m,split+j] (C is [M,split]), C2 = u when C2 != nullptr
};

struct GemmArgs {
  int M, N, K;
  const void* A; int lda; bool a_trans;
  const void* B; int ldb; bool b_trans;
  void* C; int ldc;
  int epilogue;
  const void* bias;        // [N], activation dtype
  const void* aux; int ldaux;   // [M,N] residual or pre-activation, activation dtype
  void* C2; int ldc2;      // optional second output (pre-activation u)
  void* scales;            // EPI_BIAS_RESID_ENCODE: one scale per 64 consecutive elements of C (ldc == N): fp32, or
  bool scales16;           // (scales16) bf16 bit patterns, the codes then dividing by the rounded scale
  const float* rope;       // EPI_BIAS_ROPE: (cos, sin) table [rope_S, rope_dh/2]; row m is at position m % rope_S,
  int rope_S, rope_dh, rope_cols;   // a head spans rope_dh columns, columns >= rope_cols are left alone
  int split;               // EPI_DGEGLU / EPI_BIAS_GEGLU: f, the width of the gate (and of the up) half
  float* splitk_ws;        // optional scratch of splitk_floats floats (>= gemm_splitk_floats(M, N)): lets a product with
  size_t splitk_floats;    // few output tiles and a long K be cut along K (bf16 MFMA kernel only); nullptr: never cut
  long long* stamps;       // instrumented build only: 16 int64 per workgroup of the 256 x 256 kernel (phase stamps)
};

// Floats of split-K scratch that a bf16 product with an [M, N] output can make use of (0: it is never cut).
size_t gemm_splitk_floats(int M, int N);

// T = float: plain FMA tiles (parity configuration); T = bf16: MFMA kernel.
swarm_status gemm_f32(const GemmArgs& g, hipStream_t st);
swarm_status gemm_bf16(const GemmArgs& g, hipStream_t st);
// Generic (slow, any dtype) kernel used by the fp32 path; `bf16` selects the element type.
swarm_status gemm_generic(const GemmArgs& g, bool bf16, hipStream_t st);

// ------------------------------------------------------------------ LayerNorm / reductions
// y = (x - mean) * rstd * gamma + beta over the last dim d; mean, rstd [T] fp32 are written.
swarm_status layernorm_fwd(const void* x, const void* gamma, const void* beta, void* y, float* mean, float* rstd,
                           int T, int d, float eps, bool bf16, hipStream_t st);
// dx = dres + LN-backward(dy) (dres == nullptr: no residual), dgamma += sum_t dy*xhat, dbeta += sum_t dy.
// `partial` is scratch of layernorm_bwd_scratch_floats(T, d) floats.
size_t layernorm_bwd_scratch_floats(int T, int d);
// With codes != nullptr dx is not stored: its int8 blockwise encoding is (fused stage-exit encode, bf16 and
// d % 256 == 0 only).
swarm_status layernorm_bwd(const void* dy, const void* x, const float* mean, const float* rstd, const void* gamma,
                           const void* dres, void* dx, float* dgamma, float* dbeta, float* partial, int T, int d,
                           bool bf16, hipStream_t st, int8_t* codes = nullptr, void* scales = nullptr,
                           bool scales16 = false);
// LayerNorm fused with the maxout that follows it in the compression-aware sender (k in {2, 4, 8}; other k:
// SWARM_ERR_SHAPE and nothing launched): z [T, d/k] = maxout_k(LN(x)), the normalised row is never stored.  The
// window maximum is taken on the normalised values rounded to the dtype.  k = -1: mean and rstd only.
swarm_status layernorm_fwd_maxout(const void* x, const void* gamma, const void* beta, void* z, float* mean, float* rstd,
                                  int T, int d, int k, float eps, bool bf16, hipStream_t st);
// Its backward: recomputes the normalised row from x, mean, rstd, routes dz [T, d/k] to the first maximum of every
// window and applies the LayerNorm backward; dgamma, dbeta += as in layernorm_bwd.
swarm_status layernorm_bwd_maxout(const void* dz, const void* x, const float* mean, const float* rstd,
                                  const void* gamma, const void* beta, void* dx, float* dgamma, float* dbeta,
                                  float* partial, int T, int d, int k, bool bf16, hipStream_t st);
// LayerNorm of a row that arrives int8-encoded: xdec receives the decoded row (fused stage-entry decode, bf16 only).
swarm_status layernorm_fwd_decode(const int8_t* codes, const void* scales, void* xdec, const void* gamma,
                                  const void* beta, void* y, float* mean, float* rstd, int T, int d, float eps,
                                  bool bf16, hipStream_t st, bool scales16 = false);
// Stand-alone codec launches (same kernels as the C ABI entry points).
// (scales16: the scales are bf16 bit patterns, as in swarm_codec_encode_s16 / swarm_codec_decode_s16)
swarm_status codec_decode_launch(const int8_t* codes, const void* scales, size_t n, void* tensor, bool bf16,
                                 hipStream_t st, bool scales16 = false);
swarm_status codec_encode_launch(const void* tensor, size_t n, int8_t* codes, void* scales, bool bf16,
                                 hipStream_t st, bool scales16 = false);
// out[n] += sum_t X[t,n]  (X [T,N] in the activation dtype, out fp32); scratch of colsum_scratch_floats floats.
size_t colsum_scratch_floats(int T, int N);
swarm_status colsum_accum(const void* X, int T, int N, float* out, float* partial, bool bf16, hipStream_t st);

// ------------------------------------------------------------------ rotary embedding / GeGLU
// table [S, dh/2] of (cos, sin) fp32 pairs of pos * 10000^(-2i/dh); rope_table_floats(S, dh) floats.
size_t rope_table_floats(int S, int dh);
swarm_status rope_table(float* table, int S, int dh, hipStream_t st);
// Rotates the pairs (2i, 2i+1) of every head of the q and k columns of qkv [T,3d] in place;
// inverse = rotation by the negative angle (applied to dq, dk in the backward pass).
swarm_status rope_apply(void* qkv, const float* table, int T, int S, int d, int dh, bool inverse, bool bf16,
                        hipStream_t st);
// u [T,2f] = gate | up.  g [T,f] = gelu(gate) * up.
swarm_status geglu_fwd(const void* u, void* g, int T, int f, bool bf16, hipStream_t st);
// du [T,2f] = dg * up * gelu'(gate) | dg * gelu(gate).
swarm_status geglu_bwd(const void* dg, const void* u, void* du, int T, int f, bool bf16, hipStream_t st);

// ------------------------------------------------------------------ maxout
// z[t, j] = max_{i<k} a[t, j*k + i]  (a [T, n*k] -> z [T, n]).
swarm_status maxout_fwd(const void* a, void* z, int T, int n, int k, bool bf16, hipStream_t st);
// da[t, j*k + i] = dz[t, j] for the first i with a[t, j*k+i] == max of the window, else 0.
swarm_status maxout_bwd(const void* a, const void* dz, void* da, int T, int n, int k, bool bf16, hipStream_t st);

// ------------------------------------------------------------------ attention
// qkv [T,3d] (q | k | v along the last dim; head h = columns h*dh..), causal, scores scaled by 1/sqrt(dh).
// o [T,d]; lse [B,H,S] fp32 = log-sum-exp of the scaled scores of each query row.
swarm_status attention_fwd(const void* qkv, void* o, float* lse, int B, int S, int H, int dh, bool bf16,
                           hipStream_t st);
// dqkv [T,3d] from do [T,d]; delta [B,H,S] fp32 scratch.
swarm_status attention_bwd(const void* qkv, const void* o, const void* dout, const float* lse, float* delta,
                           void* dqkv, int B, int S, int H, int dh, bool bf16, hipStream_t st);

}  // namespace swarm
