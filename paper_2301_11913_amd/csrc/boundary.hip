// Compression-aware stage-boundary layers (appendix "Compression-Aware Architectures"): host driver.
// LayerNorm, GEMM and maxout launches over a caller-provided workspace; all arithmetic is in the kernels.
#include "kernels.h"
#include "swarm_boundary.h"

namespace swarm {
namespace {

#define SWARM_TRY(expr)                 \
  do {                                  \
    swarm_status _s = (expr);           \
    if (_s != SWARM_OK) return _s;      \
  } while (0)

bool valid(const swarm_boundary_config* c) {
  if (!c) return false;
  if (c->dtype != SWARM_F32 && c->dtype != SWARM_BF16) return false;
  if (c->kind != SWARM_COMPRESS_BOTTLENECK && c->kind != SWARM_COMPRESS_MAXOUT) return false;
  if (c->d_model < 64 || c->d_model % 64 || c->d_model > 8192) return false;
  if (c->d_comp < 32 || c->d_comp % 32 || c->d_comp > c->d_model) return false;
  if (c->kind == SWARM_COMPRESS_MAXOUT && c->d_model % c->d_comp) return false;
  if (c->tokens < 1 || c->tokens > (1 << 22)) return false;
  if (!(c->ln_eps > 0.0f)) return false;
  return true;
}

struct Plan {
  void* a;          // LayerNorm output [T, w]
  void* da;         // gradient w.r.t. it (backward)
  float *mean, *rstd, *partial;
};

// w = width of the normalised tensor (m on the sender, c on the receiver)
size_t plan(const swarm_boundary_config* c, bool decompress, bool backward, void* ws, Plan& P) {
  const size_t es = c->dtype == SWARM_BF16 ? 2 : 4;
  const int w = decompress ? c->d_comp : c->d_model;
  char* base = (char*)ws;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    off = (off + 255) & ~(size_t)255;
    void* p = base ? base + off : nullptr;
    off += bytes;
    return p;
  };
  P.a = take((size_t)c->tokens * w * es);
  P.mean = (float*)take((size_t)c->tokens * 4);
  P.rstd = (float*)take((size_t)c->tokens * 4);
  P.da = nullptr; P.partial = nullptr;
  if (backward) {
    P.da = take((size_t)c->tokens * w * es);
    P.partial = (float*)take(layernorm_bwd_scratch_floats(c->tokens, w) * 4);
  }
  return (off + 255) & ~(size_t)255;
}

swarm_status gemm(bool bf16, const GemmArgs& g, hipStream_t st) { return bf16 ? gemm_bf16(g, st) : gemm_f32(g, st); }

bool al16(const void* p) { return ((uintptr_t)p & 15) == 0; }

}  // namespace
}  // namespace swarm

using namespace swarm;

extern "C" size_t swarm_boundary_workspace_bytes(const swarm_boundary_config* cfg, int decompress, int for_backward) {
  if (!valid(cfg)) return 0;
  Plan P;
  return plan(cfg, decompress != 0, for_backward != 0, nullptr, P);
}

extern "C" swarm_status swarm_compress_forward(const swarm_boundary_config* cfg, const swarm_compress_params* p,
                                               const void* y, void* z, void* workspace, size_t workspace_bytes,
                                               void* hip_stream) {
  if (!cfg || !p || !y || !z || !workspace || !p->ln_g || !p->ln_b) return SWARM_ERR_NULL;
  if (cfg->dtype != SWARM_F32 && cfg->dtype != SWARM_BF16) return SWARM_ERR_DTYPE;
  if (!valid(cfg)) return SWARM_ERR_SHAPE;
  const bool bottleneck = cfg->kind == SWARM_COMPRESS_BOTTLENECK;
  if (bottleneck && !p->w_c) return SWARM_ERR_NULL;
  if (y == z || !al16(y) || !al16(z) || ((uintptr_t)workspace & 255)) return SWARM_ERR_SHAPE;
  Plan P;
  if (plan(cfg, false, false, workspace, P) > workspace_bytes) return SWARM_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)hip_stream;
  const bool bf16 = cfg->dtype == SWARM_BF16;
  const int T = cfg->tokens, m = cfg->d_model, c = cfg->d_comp;
  if (!bottleneck) {
    // windows of 2, 4 or 8 lie inside one lane's 8 values: LayerNorm and maxout in one kernel
    const swarm_status fused = layernorm_fwd_maxout(y, p->ln_g, p->ln_b, z, P.mean, P.rstd, T, m, m / c, cfg->ln_eps,
                                                    bf16, st);
    if (fused != SWARM_ERR_SHAPE) return fused;
  }
  SWARM_TRY(layernorm_fwd(y, p->ln_g, p->ln_b, P.a, P.mean, P.rstd, T, m, cfg->ln_eps, bf16, st));
  if (!bottleneck) return maxout_fwd(P.a, z, T, c, m / c, bf16, st);
  GemmArgs g{};
  g.M = T; g.N = c; g.K = m; g.A = P.a; g.lda = m; g.B = p->w_c; g.ldb = m; g.C = z; g.ldc = c; g.epilogue = EPI_STORE;
  return gemm(bf16, g, st);
}

extern "C" swarm_status swarm_compress_backward(const swarm_boundary_config* cfg, const swarm_compress_params* p,
                                                const void* y, const void* dz, void* dy,
                                                const swarm_compress_grads* grads, void* workspace,
                                                size_t workspace_bytes, void* hip_stream) {
  if (!cfg || !p || !y || !dz || !dy || !grads || !workspace || !p->ln_g || !p->ln_b || !grads->ln_g || !grads->ln_b)
    return SWARM_ERR_NULL;
  if (cfg->dtype != SWARM_F32 && cfg->dtype != SWARM_BF16) return SWARM_ERR_DTYPE;
  if (!valid(cfg)) return SWARM_ERR_SHAPE;
  const bool bottleneck = cfg->kind == SWARM_COMPRESS_BOTTLENECK;
  if (bottleneck && (!p->w_c || !grads->w_c)) return SWARM_ERR_NULL;
  if (dy == y || dy == dz || !al16(y) || !al16(dz) || !al16(dy) || ((uintptr_t)workspace & 255)) return SWARM_ERR_SHAPE;
  Plan P;
  if (plan(cfg, false, true, workspace, P) > workspace_bytes) return SWARM_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)hip_stream;
  const bool bf16 = cfg->dtype == SWARM_BF16;
  const int T = cfg->tokens, m = cfg->d_model, c = cfg->d_comp;
  if (!bottleneck && (m / c == 2 || m / c == 4 || m / c == 8)) {
    // fused: statistics, then the LayerNorm backward that rebuilds the normalised row and routes dz itself
    SWARM_TRY(layernorm_fwd_maxout(y, p->ln_g, p->ln_b, nullptr, P.mean, P.rstd, T, m, -1, cfg->ln_eps, bf16, st));
    return layernorm_bwd_maxout(dz, y, P.mean, P.rstd, p->ln_g, p->ln_b, dy, grads->ln_g, grads->ln_b, P.partial, T, m,
                                m / c, bf16, st);
  }
  SWARM_TRY(layernorm_fwd(y, p->ln_g, p->ln_b, P.a, P.mean, P.rstd, T, m, cfg->ln_eps, bf16, st));
  if (bottleneck) {
    GemmArgs w{};   // dW_c [c, m] += dz^T a
    w.M = c; w.N = m; w.K = T; w.A = dz; w.lda = c; w.a_trans = true; w.B = P.a; w.ldb = m; w.b_trans = true;
    w.C = grads->w_c; w.ldc = m; w.epilogue = EPI_ACCUM_F32;
    SWARM_TRY(gemm(bf16, w, st));
    GemmArgs g{};   // da [T, m] = dz W_c
    g.M = T; g.N = m; g.K = c; g.A = dz; g.lda = c; g.B = p->w_c; g.ldb = m; g.b_trans = true; g.C = P.da; g.ldc = m;
    g.epilogue = EPI_STORE;
    SWARM_TRY(gemm(bf16, g, st));
  } else {
    SWARM_TRY(maxout_bwd(P.a, dz, P.da, T, c, m / c, bf16, st));
  }
  return layernorm_bwd(P.da, y, P.mean, P.rstd, p->ln_g, nullptr, dy, grads->ln_g, grads->ln_b, P.partial, T, m, bf16,
                       st);
}

extern "C" swarm_status swarm_decompress_forward(const swarm_boundary_config* cfg, const swarm_decompress_params* p,
                                                 const void* z, void* x, void* workspace, size_t workspace_bytes,
                                                 void* hip_stream) {
  if (!cfg || !p || !z || !x || !workspace || !p->ln_g || !p->ln_b || !p->w_d) return SWARM_ERR_NULL;
  if (cfg->dtype != SWARM_F32 && cfg->dtype != SWARM_BF16) return SWARM_ERR_DTYPE;
  if (!valid(cfg)) return SWARM_ERR_SHAPE;
  if (x == z || !al16(z) || !al16(x) || ((uintptr_t)workspace & 255)) return SWARM_ERR_SHAPE;
  Plan P;
  if (plan(cfg, true, false, workspace, P) > workspace_bytes) return SWARM_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)hip_stream;
  const bool bf16 = cfg->dtype == SWARM_BF16;
  const int T = cfg->tokens, m = cfg->d_model, c = cfg->d_comp;
  SWARM_TRY(layernorm_fwd(z, p->ln_g, p->ln_b, P.a, P.mean, P.rstd, T, c, cfg->ln_eps, bf16, st));
  GemmArgs g{};
  g.M = T; g.N = m; g.K = c; g.A = P.a; g.lda = c; g.B = p->w_d; g.ldb = c; g.C = x; g.ldc = m; g.epilogue = EPI_STORE;
  return gemm(bf16, g, st);
}

extern "C" swarm_status swarm_decompress_backward(const swarm_boundary_config* cfg, const swarm_decompress_params* p,
                                                  const void* z, const void* dx, void* dz,
                                                  const swarm_decompress_grads* grads, void* workspace,
                                                  size_t workspace_bytes, void* hip_stream) {
  if (!cfg || !p || !z || !dx || !dz || !grads || !workspace || !p->ln_g || !p->ln_b || !p->w_d || !grads->ln_g ||
      !grads->ln_b || !grads->w_d)
    return SWARM_ERR_NULL;
  if (cfg->dtype != SWARM_F32 && cfg->dtype != SWARM_BF16) return SWARM_ERR_DTYPE;
  if (!valid(cfg)) return SWARM_ERR_SHAPE;
  if (dz == z || dz == dx || !al16(z) || !al16(dx) || !al16(dz) || ((uintptr_t)workspace & 255)) return SWARM_ERR_SHAPE;
  Plan P;
  if (plan(cfg, true, true, workspace, P) > workspace_bytes) return SWARM_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)hip_stream;
  const bool bf16 = cfg->dtype == SWARM_BF16;
  const int T = cfg->tokens, m = cfg->d_model, c = cfg->d_comp;
  SWARM_TRY(layernorm_fwd(z, p->ln_g, p->ln_b, P.a, P.mean, P.rstd, T, c, cfg->ln_eps, bf16, st));
  GemmArgs w{};   // dW_d [m, c] += dx^T n
  w.M = m; w.N = c; w.K = T; w.A = dx; w.lda = m; w.a_trans = true; w.B = P.a; w.ldb = c; w.b_trans = true;
  w.C = grads->w_d; w.ldc = c; w.epilogue = EPI_ACCUM_F32;
  SWARM_TRY(gemm(bf16, w, st));
  GemmArgs g{};   // dn [T, c] = dx W_d
  g.M = T; g.N = c; g.K = m; g.A = dx; g.lda = m; g.B = p->w_d; g.ldb = c; g.b_trans = true; g.C = P.da; g.ldc = c;
  g.epilogue = EPI_STORE;
  SWARM_TRY(gemm(bf16, g, st));
  return layernorm_bwd(P.da, z, P.mean, P.rstd, p->ln_g, nullptr, dz, grads->ln_g, grads->ln_b, P.partial, T, c, bf16,
                       st);
}
