// Token embedding (first stage) and language-modelling head with cross-entropy (last stage): kernels and host
// driver (Section 4.3).  The embedding kernels and the softmax / loss kernels are streaming, HBM-bound; the three
// products with the vocabulary matrix go through the stage's GEMM.
#include "kernels.h"
#include "swarm_head.h"

namespace swarm {
namespace {

#define SWARM_TRY(expr)                 \
  do {                                  \
    swarm_status _s = (expr);           \
    if (_s != SWARM_OK) return _s;      \
  } while (0)

constexpr int kThreads = 256;

// 8 consecutive elements <-> fp32
template <typename T> __device__ __forceinline__ void ld8(const T* p, float (&x)[8]);
template <> __device__ __forceinline__ void ld8<bf16_raw>(const bf16_raw* p, float (&x)[8]) {
  const uint4 v = *reinterpret_cast<const uint4*>(p);
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    x[2 * i] = __uint_as_float(w[i] << 16);
    x[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
  }
}
template <> __device__ __forceinline__ void ld8<float>(const float* p, float (&x)[8]) {
  const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
  x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
}
template <typename T> __device__ __forceinline__ void st8(T* p, const float (&x)[8]);
template <> __device__ __forceinline__ void st8<bf16_raw>(bf16_raw* p, const float (&x)[8]) {
  uint4 v;
  v.x = pack_bf16x2(x[0], x[1]); v.y = pack_bf16x2(x[2], x[3]);
  v.z = pack_bf16x2(x[4], x[5]); v.w = pack_bf16x2(x[6], x[7]);
  *reinterpret_cast<uint4*>(p) = v;
}
template <> __device__ __forceinline__ void st8<float>(float* p, const float (&x)[8]) {
  *reinterpret_cast<float4*>(p) = make_float4(x[0], x[1], x[2], x[3]);
  *reinterpret_cast<float4*>(p + 4) = make_float4(x[4], x[5], x[6], x[7]);
}

// ---------------------------------------------------------------------------------------- embedding
// x[t, :] = table[token[t], :]; one thread moves 16 bytes
template <typename T>
__global__ __launch_bounds__(kThreads) void embedding_fwd_kernel(const int32_t* __restrict__ tokens,
                                                                 const T* __restrict__ table, T* __restrict__ x,
                                                                 int n_tokens, int vocab, int d) {
  constexpr int EPC = 16 / sizeof(T);          // elements per 16-byte chunk
  const int cpr = d / EPC;
  const size_t n = (size_t)n_tokens * cpr;
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += (size_t)gridDim.x * kThreads) {
    const int t = (int)(i / cpr), c = (int)(i - (size_t)t * cpr);
    const int id = tokens[t];
    uint4 v = make_uint4(0, 0, 0, 0);
    if (id >= 0 && id < vocab) v = *reinterpret_cast<const uint4*>(table + (size_t)id * d + c * EPC);
    *reinterpret_cast<uint4*>(x + (size_t)t * d + c * EPC) = v;
  }
}

// grad_table[id, :] += sum over positions t' with token[t'] == id of dx[t', :], in increasing t'.
// The workgroups (t, y) do the whole sum (each for its own 2048 columns) if t is the first position of its id,
// otherwise nothing: no two workgroups touch the same elements, no atomics.  Positions are scanned 256 at a time; the matches of a round are put into LDS in
// position order (wave ballots + popcounts), then every thread adds those rows to its own columns.
template <typename T>
__global__ __launch_bounds__(kThreads) void embedding_bwd_kernel(const int32_t* __restrict__ tokens,
                                                                 const T* __restrict__ dx, float* __restrict__ grad,
                                                                 int n_tokens, int vocab, int d) {
  __shared__ int s_list[kThreads];
  __shared__ int s_wave_cnt[kThreads / 64];
  __shared__ int s_flag;
  const int t0 = blockIdx.x;
  const int id = tokens[t0];
  if (id < 0 || id >= vocab) return;
  if (threadIdx.x == 0) s_flag = 0;
  __syncthreads();
  int seen = 0;
  for (int t = threadIdx.x; t < t0; t += kThreads) seen |= tokens[t] == id;
  if (seen) s_flag = 1;          // benign race: every writer stores 1
  __syncthreads();
  if (s_flag) return;

  // blockIdx.y picks this workgroup's 256 column chunks of 8 (a frequent id has hundreds of rows to add: the
  // columns are spread over several workgroups and the row loads go out eight at a time)
  const int c = blockIdx.y * kThreads + threadIdx.x;
  const bool live = c < (d >> 3);
  float acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = 0.f;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int base = t0; base < n_tokens; base += kThreads) {
    const int t = base + threadIdx.x;
    const bool match = t < n_tokens && tokens[t] == id;
    const unsigned long long ballot = __ballot(match);
    if (lane == 0) s_wave_cnt[wave] = __popcll(ballot);
    __syncthreads();
    int before = 0, total = 0;
#pragma unroll
    for (int w = 0; w < kThreads / 64; ++w) {
      if (w < wave) before += s_wave_cnt[w];
      total += s_wave_cnt[w];
    }
    if (match) s_list[before + __popcll(ballot & ((1ull << lane) - 1ull))] = t;
    __syncthreads();
    if (live) {
      constexpr int U = 8;
      for (int j0 = 0; j0 < total; j0 += U) {
        float v[U][8];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int j = min(j0 + u, total - 1);            // past the end: a re-read that is not added
          ld8<T>(dx + (size_t)s_list[j] * d + c * 8, v[u]);
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
          if (j0 + u < total) {
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] += v[u][e];
          }
      }
    }
    __syncthreads();             // s_list and s_wave_cnt are rewritten by the next round
  }
  if (live) {
    float* out = grad + (size_t)id * d + c * 8;
#pragma unroll
    for (int e = 0; e < 8; ++e) out[e] += acc[e];
  }
}

// ---------------------------------------------------------------------------------------- softmax cross-entropy
// One workgroup per token row of logits [T, ld] (columns >= vocab are padding).  Pass 1: running maximum and sum of
// exponentials (online, one read); token_loss = log(sum) + max - logit[target].  GRAD: pass 2 overwrites the row
// with (softmax - onehot) * inv_T, zeros in the padding.
template <typename T, bool GRAD>
__global__ __launch_bounds__(kThreads) void softmax_ce_kernel(T* __restrict__ logits, const int32_t* __restrict__ targets,
                                                             float* __restrict__ token_loss, int vocab, int ld,
                                                             float inv_T) {
  __shared__ float s_m[kThreads / 64], s_s[kThreads / 64];
  T* row = logits + (size_t)blockIdx.x * ld;
  float m = -INFINITY, s = 0.f;
  for (int c = threadIdx.x; c * 8 < vocab; c += kThreads) {     // rows are 8-element aligned (ld % 8 == 0)
    float l[8];
    ld8<T>(row + c * 8, l);
    float cm = -INFINITY;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      if (c * 8 + e >= vocab) l[e] = -INFINITY;
      cm = fmaxf(cm, l[e]);
    }
    if (cm > m) { s *= __expf(m - cm); m = cm; }
#pragma unroll
    for (int e = 0; e < 8; ++e) s += __expf(l[e] - m);          // exp(-inf) = 0 for the padding
  }
  // combine (m, s) pairs: lanes, then wavefronts, in a fixed order
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const float mo = __shfl_xor(m, off, 64), so = __shfl_xor(s, off, 64);
    const float mn = fmaxf(m, mo);
    s = (m == -INFINITY ? 0.f : s * __expf(m - mn)) + (mo == -INFINITY ? 0.f : so * __expf(mo - mn));
    m = mn;
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (lane == 0) { s_m[wave] = m; s_s[wave] = s; }
  __syncthreads();
  m = s_m[0]; s = s_s[0];
#pragma unroll
  for (int w = 1; w < kThreads / 64; ++w) {
    const float mo = s_m[w], so = s_s[w];
    const float mn = fmaxf(m, mo);
    s = (m == -INFINITY ? 0.f : s * __expf(m - mn)) + (mo == -INFINITY ? 0.f : so * __expf(mo - mn));
    m = mn;
  }
  const float lse = logf(s) + m;
  const int tgt = targets[blockIdx.x];
  const bool tgt_ok = tgt >= 0 && tgt < vocab;
  if (threadIdx.x == 0) token_loss[blockIdx.x] = lse - (tgt_ok ? Elem<T>::load(row + tgt) : 0.f);
  if constexpr (GRAD) {
    __syncthreads();             // the target logit has been read before the row is overwritten
    for (int c = threadIdx.x; c * 8 < ld; c += kThreads) {
      float l[8], g[8];
      ld8<T>(row + c * 8, l);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int v = c * 8 + e;
        g[e] = v < vocab ? (__expf(l[e] - lse) - (v == tgt ? 1.f : 0.f)) * inv_T : 0.f;
      }
      st8<T>(row + c * 8, g);
    }
  }
}

// loss = (sum of the token losses, fixed order) / T; one workgroup
__global__ __launch_bounds__(kThreads) void mean_kernel(const float* __restrict__ v, int n, float* __restrict__ out) {
  __shared__ float s_p[kThreads];
  float a = 0.f;
  for (int i = threadIdx.x; i < n; i += kThreads) a += v[i];
  s_p[threadIdx.x] = a;
  __syncthreads();
  for (int w = kThreads / 2; w >= 1; w >>= 1) {
    if (threadIdx.x < w) s_p[threadIdx.x] += s_p[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) *out = s_p[0] / (float)n;
}

bool valid(const swarm_head_config* c) {
  if (!c) return false;
  if (c->dtype != SWARM_F32 && c->dtype != SWARM_BF16) return false;
  if (c->d_model < 64 || c->d_model % 64 || c->d_model > 8192) return false;
  if (c->vocab < 1 || c->vocab_rows < c->vocab || c->vocab_rows % 8) return false;
  if (c->tokens < 1 || c->tokens > (1 << 22)) return false;
  if ((long long)c->tokens * c->vocab_rows > (1ll << 34)) return false;
  if (!(c->ln_eps > 0.0f)) return false;
  return true;
}

struct Plan {
  void *n, *logits, *dn;
  float *mean, *rstd, *tok, *partial;
  float* splitk;
  size_t splitk_floats;
};

size_t plan(const swarm_head_config* c, bool backward, void* ws, Plan& P) {
  const size_t es = c->dtype == SWARM_BF16 ? 2 : 4;
  char* base = (char*)ws;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    off = (off + 255) & ~(size_t)255;
    void* p = base ? base + off : nullptr;
    off += bytes;
    return p;
  };
  const size_t T = c->tokens;
  P.n = take(T * c->d_model * es);
  P.mean = (float*)take(T * 4);
  P.rstd = (float*)take(T * 4);
  P.tok = (float*)take(T * 4);
  P.logits = take(T * c->vocab_rows * es);
  P.dn = nullptr; P.partial = nullptr; P.splitk = nullptr; P.splitk_floats = 0;
  if (backward) {
    P.dn = take(T * c->d_model * es);
    P.partial = (float*)take(layernorm_bwd_scratch_floats(c->tokens, c->d_model) * 4);
    // dn = dlogits W has few output tiles and K = vocabulary rows: scratch for cutting it along K
    P.splitk_floats = c->dtype == SWARM_BF16 ? gemm_splitk_floats(c->tokens, c->d_model) : 0;
    if (P.splitk_floats) P.splitk = (float*)take(P.splitk_floats * 4);
  }
  return (off + 255) & ~(size_t)255;
}

swarm_status gemm(bool bf16, const GemmArgs& g, hipStream_t st) { return bf16 ? gemm_bf16(g, st) : gemm_f32(g, st); }
bool al16(const void* p) { return ((uintptr_t)p & 15) == 0; }

swarm_status run_head(const swarm_head_config* cfg, const swarm_head_params* p, const void* x, const int32_t* targets,
                      float* loss, float* token_loss, void* dx, const swarm_head_grads* grads, const Plan& P,
                      hipStream_t st) {
  const bool bf16 = cfg->dtype == SWARM_BF16, backward = dx != nullptr;
  const int T = cfg->tokens, d = cfg->d_model, Vp = cfg->vocab_rows;
  SWARM_TRY(layernorm_fwd(x, p->ln_g, p->ln_b, P.n, P.mean, P.rstd, T, d, cfg->ln_eps, bf16, st));
  GemmArgs l{};   // logits [T, Vp] = n W^T
  l.M = T; l.N = Vp; l.K = d; l.A = P.n; l.lda = d; l.B = p->w_vocab; l.ldb = d; l.C = P.logits; l.ldc = Vp;
  l.epilogue = EPI_STORE;
  SWARM_TRY(gemm(bf16, l, st));
  float* tok = token_loss ? token_loss : P.tok;
  const float inv_T = 1.0f / (float)T;
  if (bf16) {
    if (backward)
      hipLaunchKernelGGL((softmax_ce_kernel<bf16_raw, true>), dim3(T), dim3(kThreads), 0, st, (bf16_raw*)P.logits,
                         targets, tok, cfg->vocab, Vp, inv_T);
    else
      hipLaunchKernelGGL((softmax_ce_kernel<bf16_raw, false>), dim3(T), dim3(kThreads), 0, st, (bf16_raw*)P.logits,
                         targets, tok, cfg->vocab, Vp, inv_T);
  } else {
    if (backward)
      hipLaunchKernelGGL((softmax_ce_kernel<float, true>), dim3(T), dim3(kThreads), 0, st, (float*)P.logits, targets,
                         tok, cfg->vocab, Vp, inv_T);
    else
      hipLaunchKernelGGL((softmax_ce_kernel<float, false>), dim3(T), dim3(kThreads), 0, st, (float*)P.logits, targets,
                         tok, cfg->vocab, Vp, inv_T);
  }
  hipLaunchKernelGGL(mean_kernel, dim3(1), dim3(kThreads), 0, st, tok, T, loss);
  SWARM_TRY(launch_status());
  if (!backward) return SWARM_OK;
  GemmArgs w{};   // dW [Vp, d] += dlogits^T n   (padding rows receive +0)
  w.M = Vp; w.N = d; w.K = T; w.A = P.logits; w.lda = Vp; w.a_trans = true; w.B = P.n; w.ldb = d; w.b_trans = true;
  w.C = grads->w_vocab; w.ldc = d; w.epilogue = EPI_ACCUM_F32;
  SWARM_TRY(gemm(bf16, w, st));
  GemmArgs g{};   // dn [T, d] = dlogits W
  g.M = T; g.N = d; g.K = Vp; g.A = P.logits; g.lda = Vp; g.B = p->w_vocab; g.ldb = d; g.b_trans = true; g.C = P.dn;
  g.ldc = d; g.epilogue = EPI_STORE; g.splitk_ws = P.splitk; g.splitk_floats = P.splitk_floats;
  SWARM_TRY(gemm(bf16, g, st));
  return layernorm_bwd(P.dn, x, P.mean, P.rstd, p->ln_g, nullptr, dx, grads->ln_g, grads->ln_b, P.partial, T, d, bf16,
                       st);
}

}  // namespace
}  // namespace swarm

using namespace swarm;

extern "C" swarm_status swarm_embedding_forward(const int32_t* tokens, const void* table, int32_t dtype,
                                                int32_t n_tokens, int32_t vocab, int32_t d_model, void* x,
                                                void* hip_stream) {
  if (!tokens || !table || !x) return SWARM_ERR_NULL;
  if (dtype != SWARM_F32 && dtype != SWARM_BF16) return SWARM_ERR_DTYPE;
  if (n_tokens < 1 || vocab < 1 || d_model < 8 || d_model % 8 || !al16(table) || !al16(x)) return SWARM_ERR_SHAPE;
  hipStream_t st = (hipStream_t)hip_stream;
  const size_t chunks = (size_t)n_tokens * (d_model / (dtype == SWARM_BF16 ? 8 : 4));
  const int grid = (int)std::min<size_t>((chunks + kThreads - 1) / kThreads, 256 * 16);
  if (dtype == SWARM_BF16)
    hipLaunchKernelGGL(embedding_fwd_kernel<bf16_raw>, dim3(grid), dim3(kThreads), 0, st, tokens,
                       (const bf16_raw*)table, (bf16_raw*)x, n_tokens, vocab, d_model);
  else
    hipLaunchKernelGGL(embedding_fwd_kernel<float>, dim3(grid), dim3(kThreads), 0, st, tokens, (const float*)table,
                       (float*)x, n_tokens, vocab, d_model);
  return launch_status();
}

extern "C" swarm_status swarm_embedding_backward(const int32_t* tokens, const void* dx, int32_t dtype,
                                                 int32_t n_tokens, int32_t vocab, int32_t d_model, float* grad_table,
                                                 void* hip_stream) {
  if (!tokens || !dx || !grad_table) return SWARM_ERR_NULL;
  if (dtype != SWARM_F32 && dtype != SWARM_BF16) return SWARM_ERR_DTYPE;
  if (n_tokens < 1 || n_tokens > 65536 || vocab < 1 || d_model < 8 || d_model % 8 || d_model > 8192 || !al16(dx))
    return SWARM_ERR_SHAPE;
  hipStream_t st = (hipStream_t)hip_stream;
  const dim3 grid(n_tokens, (d_model / 8 + kThreads - 1) / kThreads);
  if (dtype == SWARM_BF16)
    hipLaunchKernelGGL(embedding_bwd_kernel<bf16_raw>, grid, dim3(kThreads), 0, st, tokens,
                       (const bf16_raw*)dx, grad_table, n_tokens, vocab, d_model);
  else
    hipLaunchKernelGGL(embedding_bwd_kernel<float>, grid, dim3(kThreads), 0, st, tokens, (const float*)dx,
                       grad_table, n_tokens, vocab, d_model);
  return launch_status();
}

extern "C" size_t swarm_head_workspace_bytes(const swarm_head_config* cfg, int for_backward) {
  if (!valid(cfg)) return 0;
  Plan P;
  return plan(cfg, for_backward != 0, nullptr, P);
}

extern "C" swarm_status swarm_head_loss(const swarm_head_config* cfg, const swarm_head_params* p, const void* x,
                                        const int32_t* targets, float* loss, float* token_loss, void* workspace,
                                        size_t workspace_bytes, void* hip_stream) {
  if (!cfg || !p || !x || !targets || !loss || !workspace || !p->ln_g || !p->ln_b || !p->w_vocab) return SWARM_ERR_NULL;
  if (cfg->dtype != SWARM_F32 && cfg->dtype != SWARM_BF16) return SWARM_ERR_DTYPE;
  if (!valid(cfg)) return SWARM_ERR_SHAPE;
  if (!al16(x) || ((uintptr_t)workspace & 255)) return SWARM_ERR_SHAPE;
  Plan P;
  if (plan(cfg, false, workspace, P) > workspace_bytes) return SWARM_ERR_WORKSPACE;
  return run_head(cfg, p, x, targets, loss, token_loss, nullptr, nullptr, P, (hipStream_t)hip_stream);
}

extern "C" swarm_status swarm_head_loss_backward(const swarm_head_config* cfg, const swarm_head_params* p,
                                                 const void* x, const int32_t* targets, float* loss,
                                                 float* token_loss, void* dx, const swarm_head_grads* grads,
                                                 void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!cfg || !p || !x || !targets || !loss || !dx || !grads || !workspace || !p->ln_g || !p->ln_b || !p->w_vocab ||
      !grads->ln_g || !grads->ln_b || !grads->w_vocab)
    return SWARM_ERR_NULL;
  if (cfg->dtype != SWARM_F32 && cfg->dtype != SWARM_BF16) return SWARM_ERR_DTYPE;
  if (!valid(cfg)) return SWARM_ERR_SHAPE;
  if (dx == x || !al16(x) || !al16(dx) || ((uintptr_t)workspace & 255)) return SWARM_ERR_SHAPE;
  Plan P;
  if (plan(cfg, true, workspace, P) > workspace_bytes) return SWARM_ERR_WORKSPACE;
  return run_head(cfg, p, x, targets, loss, token_loss, dx, grads, P, (hipStream_t)hip_stream);
}
