// Stage driver: the fixed sequence of kernel launches for one pipeline stage's forward and
// checkpoint-recomputing backward (paper Section 3.2), plus workspace carving and argument
// validation.  Host code only; all arithmetic happens in the kernels it launches.
#include <algorithm>
#include <cstdlib>

#include "kernels.h"

namespace swarm {

swarm_status attention_fwd_naive(const void*, void*, float*, int, int, int, int, bool, hipStream_t);
swarm_status attention_bwd_naive(const void*, const void*, const void*, const float*, float*, void*, int, int, int,
                                 int, bool, hipStream_t);

namespace {

struct Dims {
  int T, d, f, H, dh, B, S, apps;
  int f1;     // rows of w_1: f, or 2f (gate | up) for the rotary + GeGLU block
  bool rope_geglu;
  bool bf16;
  size_t es;  // element size of the activation dtype
  float* splitk = nullptr;      // split-K scratch for the bf16 products with few output tiles (set once the
  size_t splitk_floats = 0;     // workspace is carved)
};

// split-K scratch that the products of this configuration can use: the widest of their four output shapes
size_t splitk_floats_of(const Dims& D) {
  if (!D.bf16) return 0;
  return std::max(std::max(gemm_splitk_floats(D.T, D.d), gemm_splitk_floats(D.T, 3 * D.d)),
                  std::max(gemm_splitk_floats(D.T, D.f), gemm_splitk_floats(D.T, D.f1)));
}

bool valid_config(const swarm_stage_config* c) {
  if (!c) return false;
  if (c->dtype != SWARM_F32 && c->dtype != SWARM_BF16) return false;
  if (c->d_model < 64 || c->d_model % 64 || c->d_ffn < 64 || c->d_ffn % 64) return false;
  if (c->d_model > 8192) return false;
  if (c->n_heads < 1 || c->d_model % c->n_heads) return false;
  const int dh = c->d_model / c->n_heads;
  if (dh != 64 && dh != 128) return false;
  if (c->n_layers < 1 || c->n_repeat < 1 || c->batch < 1 || c->seq < 1) return false;
  if ((long long)c->batch * c->seq > (1ll << 24)) return false;
  if (c->seq > 7000 && c->dtype == SWARM_F32) return false;   // direct attention keeps a score row in LDS
  if (!(c->ln_eps > 0.0f)) return false;
  if (c->block_kind != SWARM_BLOCK_GELU && c->block_kind != SWARM_BLOCK_ROTARY_GEGLU) return false;
  return true;
}

Dims dims_of(const swarm_stage_config* c) {
  Dims D;
  D.B = c->batch; D.S = c->seq; D.T = c->batch * c->seq; D.d = c->d_model; D.f = c->d_ffn; D.H = c->n_heads;
  D.dh = D.d / D.H; D.apps = c->n_layers * c->n_repeat; D.bf16 = c->dtype == SWARM_BF16;
  D.es = D.bf16 ? 2 : 4;
  D.rope_geglu = c->block_kind == SWARM_BLOCK_ROTARY_GEGLU;
  D.f1 = D.rope_geglu ? 2 * D.f : D.f;
  return D;
}

// Bump allocator over the caller's workspace; with base == nullptr it only measures.
struct Carver {
  char* base;
  size_t off = 0;
  explicit Carver(void* b) : base((char*)b) {}
  void* take(size_t bytes) {
    off = (off + 255) & ~(size_t)255;
    void* p = base ? base + off : nullptr;
    off += bytes;
    return p;
  }
  size_t total() const { return (off + 255) & ~(size_t)255; }
};

// Intermediates of one block application.
struct Saved {
  const void* x;   // block input [T,d]
  void *a, *qkv, *o, *h, *c, *u, *g;
  float *mean1, *rstd1, *mean2, *rstd2, *lse;
  const float* rope;   // (cos, sin) table shared by all applications; nullptr for the GeLU block
};

void carve_saved(Carver& cv, const Dims& D, Saved& s, bool want_u) {
  const size_t Td = (size_t)D.T * D.d * D.es, Tf = (size_t)D.T * D.f * D.es;
  s.a = cv.take(Td); s.qkv = cv.take(3 * Td); s.o = cv.take(Td); s.h = cv.take(Td); s.c = cv.take(Td);
  // the GeGLU block always materialises u = gate | up; the GeLU block needs u only for the backward pass
  s.u = (want_u || D.rope_geglu) ? cv.take((size_t)D.T * D.f1 * D.es) : nullptr;
  s.g = cv.take(Tf);
  s.mean1 = (float*)cv.take((size_t)D.T * 4); s.rstd1 = (float*)cv.take((size_t)D.T * 4);
  s.mean2 = (float*)cv.take((size_t)D.T * 4); s.rstd2 = (float*)cv.take((size_t)D.T * 4);
  s.lse = (float*)cv.take((size_t)D.B * D.H * D.S * 4);
}

swarm_status gemm(const Dims& D, const GemmArgs& g, hipStream_t st) {
  if (!D.bf16) return gemm_f32(g, st);
  GemmArgs h = g;
  h.splitk_ws = D.splitk; h.splitk_floats = D.splitk_floats;
  return gemm_bf16(h, st);
}

#define SWARM_TRY(expr)                 \
  do {                                  \
    swarm_status _s = (expr);           \
    if (_s != SWARM_OK) return _s;      \
  } while (0)

// Stage-boundary codec fused into a block: `in_codes` -> the block input arrives int8-encoded and is decoded
// into s.x by LN1; `out_codes` -> the block output leaves int8-encoded from the FFN2 epilogue.
struct Boundary {
  const int8_t* in_codes = nullptr; const void* in_scales = nullptr;
  int8_t* out_codes = nullptr; void* out_scales = nullptr;
  bool scales16 = false;   // block scales are bf16 bit patterns instead of fp32
};

// y = block(x): writes every intermediate into `s`; the last GEMM is skipped when y == nullptr.
swarm_status block_forward(const Dims& D, const swarm_block_params& p, const Saved& s, void* y, float eps,
                           hipStream_t st, const Boundary& bd = Boundary(), bool want_u = true) {
  const int T = D.T, d = D.d, f = D.f;
  if (bd.in_codes)
    SWARM_TRY(layernorm_fwd_decode(bd.in_codes, bd.in_scales, const_cast<void*>(s.x), p.ln1_g, p.ln1_b, s.a, s.mean1,
                                   s.rstd1, T, d, eps, D.bf16, st, bd.scales16));
  else
    SWARM_TRY(layernorm_fwd(s.x, p.ln1_g, p.ln1_b, s.a, s.mean1, s.rstd1, T, d, eps, D.bf16, st));
  GemmArgs q{};
  q.M = T; q.N = 3 * d; q.K = d; q.A = s.a; q.lda = d; q.B = p.w_qkv; q.ldb = d; q.C = s.qkv; q.ldc = 3 * d;
  q.epilogue = EPI_BIAS; q.bias = p.b_qkv;
  if (D.rope_geglu) {
    // rotary in the QKV epilogue (fp32, before the rounding to bf16) where the MFMA GEMM takes the shape
    swarm_status fused = SWARM_ERR_SHAPE;
    if (D.bf16) {
      GemmArgs qr = q;
      qr.epilogue = EPI_BIAS_ROPE; qr.rope = s.rope; qr.rope_S = D.S; qr.rope_dh = D.dh; qr.rope_cols = 2 * d;
      fused = gemm(D, qr, st);
    }
    if (fused == SWARM_ERR_SHAPE) {
      SWARM_TRY(gemm(D, q, st));
      SWARM_TRY(rope_apply(s.qkv, s.rope, T, D.S, d, D.dh, false, D.bf16, st));
    } else {
      SWARM_TRY(fused);
    }
  } else {
    SWARM_TRY(gemm(D, q, st));
  }
  SWARM_TRY(attention_fwd(s.qkv, s.o, s.lse, D.B, D.S, D.H, D.dh, D.bf16, st));
  GemmArgs o{};
  o.M = T; o.N = d; o.K = d; o.A = s.o; o.lda = d; o.B = p.w_o; o.ldb = d; o.C = s.h; o.ldc = d;
  o.epilogue = EPI_BIAS_RESID; o.bias = p.b_o; o.aux = s.x; o.ldaux = d;
  SWARM_TRY(gemm(D, o, st));
  SWARM_TRY(layernorm_fwd(s.h, p.ln2_g, p.ln2_b, s.c, s.mean2, s.rstd2, T, d, eps, D.bf16, st));
  GemmArgs f1{};
  f1.M = T; f1.N = f; f1.K = d; f1.A = s.c; f1.lda = d; f1.B = p.w_1; f1.ldb = d; f1.C = s.g; f1.ldc = f;
  f1.epilogue = EPI_BIAS_GELU; f1.bias = p.b_1; f1.C2 = s.u; f1.ldc2 = f;
  if (D.rope_geglu) {
    // gate * up in the FFN1 epilogue (u = gate | up is stored only when the caller keeps it for the backward)
    swarm_status fused = SWARM_ERR_SHAPE;
    if (D.bf16) {
      GemmArgs fg = f1;
      fg.N = 2 * f; fg.epilogue = EPI_BIAS_GEGLU; fg.split = f; fg.C2 = want_u ? s.u : nullptr; fg.ldc2 = 2 * f;
      fused = gemm(D, fg, st);
    }
    if (fused == SWARM_ERR_SHAPE) {
      f1.N = 2 * f; f1.C = s.u; f1.ldc = 2 * f; f1.epilogue = EPI_BIAS; f1.C2 = nullptr;
      SWARM_TRY(gemm(D, f1, st));
      SWARM_TRY(geglu_fwd(s.u, s.g, T, f, D.bf16, st));
    } else {
      SWARM_TRY(fused);
    }
  } else {
    SWARM_TRY(gemm(D, f1, st));
  }
  if (y || bd.out_codes) {
    GemmArgs f2{};
    f2.M = T; f2.N = d; f2.K = f; f2.A = s.g; f2.lda = f; f2.B = p.w_2; f2.ldb = f; f2.C = y; f2.ldc = d;
    f2.epilogue = EPI_BIAS_RESID; f2.bias = p.b_2; f2.aux = s.h; f2.ldaux = d;
    if (bd.out_codes) {
      f2.epilogue = EPI_BIAS_RESID_ENCODE; f2.C = bd.out_codes; f2.scales = bd.out_scales; f2.scales16 = bd.scales16;
    }
    SWARM_TRY(gemm(D, f2, st));
  }
  return SWARM_OK;
}

// Scratch of one block_backward call (reused by every application).
struct BwdTemps {
  void *dc, *dout, *da;
  void* dg;   // GeGLU block only: gradient of g [T,f]
  float *delta, *partial;
};

// Gradients that feed the weight-gradient GEMMs of one application: the gradient of the block output (dy, given),
// of the FFN pre-activation (du), of the hidden stream (dh) and of q|k|v (dqkv).  The applications of one
// parameter set keep theirs in consecutive slots, so that the set's weight gradients are ONE product over all
// its tokens (see set_weight_grads).
struct AppGrads {
  void *du, *dh, *dqkv;
};

// dW[out,in] += dY^T X  and  db[out] += colsum(dY)  over `rows` token rows
swarm_status weight_grads(const Dims& D, int rows, const void* dY, int n_out, const void* X, int n_in, float* dW,
                          float* db, float* partial, hipStream_t st) {
  SWARM_TRY(colsum_accum(dY, rows, n_out, db, partial, D.bf16, st));
  GemmArgs w{};
  w.M = n_out; w.N = n_in; w.K = rows; w.A = dY; w.lda = n_out; w.a_trans = true; w.B = X; w.ldb = n_in;
  w.b_trans = true; w.C = dW; w.ldc = n_in; w.epilogue = EPI_ACCUM_F32;
  return gemm(D, w, st);
}

// dX[T,in] = dY[T,out] W[out,in]
swarm_status data_grad(const Dims& D, const void* dY, int n_out, const void* W, int n_in, void* dX, int epilogue,
                       const void* aux, hipStream_t st) {
  GemmArgs g{};
  g.M = D.T; g.N = n_in; g.K = n_out; g.A = dY; g.lda = n_out; g.B = W; g.ldb = n_in; g.b_trans = true;
  g.C = dX; g.ldc = n_in; g.epilogue = epilogue; g.aux = aux; g.ldaux = n_in;
  return gemm(D, g, st);
}

// Data gradients and LayerNorm parameter gradients of one application; the matrix weight / bias gradients are
// left to set_weight_grads, which reads dy and the tensors stored in `ag`.
swarm_status block_backward(const Dims& D, const swarm_block_params& p, const swarm_block_grads& gp, const Saved& s,
                            const BwdTemps& t, const AppGrads& ag, const void* dy, void* dx, hipStream_t st,
                            int8_t* dx_codes = nullptr, void* dx_scales = nullptr, bool scales16 = false) {
  const int d = D.d, f = D.f;
  // y = h + g W2^T + b2,  g = gelu(u)  or  gelu(u_gate) * u_up
  if (D.rope_geglu) {
    // du = (dg * up * gelu'(gate) | dg * gelu(gate)) in the epilogue of dg = dy W2
    swarm_status fused = SWARM_ERR_SHAPE;
    if (D.bf16) {
      GemmArgs g{};
      g.M = D.T; g.N = f; g.K = d; g.A = dy; g.lda = d; g.B = p.w_2; g.ldb = f; g.b_trans = true;
      g.C = ag.du; g.ldc = 2 * f; g.epilogue = EPI_DGEGLU; g.aux = s.u; g.ldaux = 2 * f; g.split = f;
      fused = gemm(D, g, st);
    }
    if (fused == SWARM_ERR_SHAPE) {
      SWARM_TRY(data_grad(D, dy, d, p.w_2, f, t.dg, EPI_STORE, nullptr, st));
      SWARM_TRY(geglu_bwd(t.dg, s.u, ag.du, D.T, f, D.bf16, st));
    } else {
      SWARM_TRY(fused);
    }
  } else {
    SWARM_TRY(data_grad(D, dy, d, p.w_2, f, ag.du, EPI_DGELU, s.u, st));
  }
  // u = c W1^T + b1
  SWARM_TRY(data_grad(D, ag.du, D.f1, p.w_1, d, t.dc, EPI_STORE, nullptr, st));
  // c = LN2(h);  dh = dy + LN2'(dc)
  SWARM_TRY(layernorm_bwd(t.dc, s.h, s.mean2, s.rstd2, p.ln2_g, dy, ag.dh, gp.ln2_g, gp.ln2_b, t.partial, D.T, d,
                          D.bf16, st));
  // h = x + o Wo^T + bo
  SWARM_TRY(data_grad(D, ag.dh, d, p.w_o, d, t.dout, EPI_STORE, nullptr, st));
  SWARM_TRY(attention_bwd(s.qkv, s.o, t.dout, s.lse, t.delta, ag.dqkv, D.B, D.S, D.H, D.dh, D.bf16, st));
  // the saved q, k are the rotated ones: turn their gradients back
  if (D.rope_geglu) SWARM_TRY(rope_apply(ag.dqkv, s.rope, D.T, D.S, d, D.dh, true, D.bf16, st));
  // qkv = a Wqkv^T + bqkv
  SWARM_TRY(data_grad(D, ag.dqkv, 3 * d, p.w_qkv, d, t.da, EPI_STORE, nullptr, st));
  // a = LN1(x);  dx = dh + LN1'(da)
  SWARM_TRY(layernorm_bwd(t.da, s.x, s.mean1, s.rstd1, p.ln1_g, ag.dh, dx, gp.ln1_g, gp.ln1_b, t.partial, D.T, d,
                          D.bf16, st, dx_codes, dx_scales, scales16));
  return SWARM_OK;
}

// Weight and bias gradients of one parameter set over `n` consecutive applications whose tensors start at the
// given pointers (slot pitch = one application's tensor): with layer sharing (Sections 2.3 and 4.3) the sum over
// the applications is the K dimension of a single product, dW += [dY_0; ...; dY_{n-1}]^T [X_0; ...; X_{n-1}],
// so the fp32 gradient matrix is read and written once per set instead of once per application.
swarm_status set_weight_grads(const Dims& D, const swarm_block_grads& gp, int n, const void* dy, const AppGrads& ag,
                              const Saved& s, float* partial, hipStream_t st) {
  const int rows = n * D.T, d = D.d;
  SWARM_TRY(weight_grads(D, rows, dy, d, s.g, D.f, gp.w_2, gp.b_2, partial, st));
  SWARM_TRY(weight_grads(D, rows, ag.du, D.f1, s.c, d, gp.w_1, gp.b_1, partial, st));
  SWARM_TRY(weight_grads(D, rows, ag.dh, d, s.o, d, gp.w_o, gp.b_o, partial, st));
  SWARM_TRY(weight_grads(D, rows, ag.dqkv, 3 * d, s.a, d, gp.w_qkv, gp.b_qkv, partial, st));
  return SWARM_OK;
}

struct FwdPlan {
  Saved s;
  void* z[2];
  float* rope;
  float* splitk;
};

size_t plan_forward(const Dims& D, void* ws, FwdPlan& P) {
  Carver cv(ws);
  const size_t Td = (size_t)D.T * D.d * D.es;
  P.s = Saved{};
  carve_saved(cv, D, P.s, false);
  P.rope = D.rope_geglu ? (float*)cv.take(rope_table_floats(D.S, D.dh) * 4) : nullptr;
  P.s.rope = P.rope;
  P.z[0] = D.apps > 1 ? cv.take(Td) : nullptr;
  P.z[1] = D.apps > 1 ? cv.take(Td) : nullptr;
  P.splitk = splitk_floats_of(D) ? (float*)cv.take(splitk_floats_of(D) * 4) : nullptr;
  return cv.total();
}

// Token rows per weight-gradient product (a longer run of shared applications is cut into several products).
constexpr long long kMaxWgradRows = 1ll << 22;

int wgrad_chunk(const Dims& D, int R) {
  return (int)std::max<long long>(1, std::min<long long>(R, kMaxWgradRows / D.T));
}

// Workspace layout of the backward call.  Plain pointers and pitches only: the plan lives on the caller's stack and
// the intermediates of application i are found by arithmetic (saved_at), so a call touches no host heap.
struct BwdPlan {
  char *a_all, *o_all, *c_all, *g_all;   // [apps] slots of [T,d] x3 and [T,f]: right-hand operands of the wgrads
  char* app_slots;                        // [apps] slots of app_pitch bytes: qkv, h, u, row statistics, lse, input
  size_t app_pitch, off_h, off_u, off_stats, off_lse, off_x;
  BwdTemps t;
  char *du_slots, *dh_slots, *dqkv_slots;   // [R] slots of [T,f1], [T,d], [T,3d]: one per application of a set
  char* dys[2];              // [R] slots of [T,d] (gradient of each application's output), by parameter-set parity
  float* rope;
  float* splitk;
};

size_t plan_backward(const Dims& D, int L, int R, void* ws, BwdPlan& P) {
  Carver cv(ws);
  const size_t Td = (size_t)D.T * D.d * D.es, Tf = (size_t)D.T * D.f * D.es, Tf1 = (size_t)D.T * D.f1 * D.es;
  P.rope = D.rope_geglu ? (float*)cv.take(rope_table_floats(D.S, D.dh) * 4) : nullptr;
  // the right-hand operands of the weight-gradient products are contiguous over the applications
  P.a_all = (char*)cv.take(D.apps * Td);
  P.o_all = (char*)cv.take(D.apps * Td);
  P.c_all = (char*)cv.take(D.apps * Td);
  P.g_all = (char*)cv.take(D.apps * Tf);
  {
    Carver slot(nullptr);   // one application's private tensors, measured once; every slot has the same layout
    slot.take(3 * Td);
    slot.take(Td); P.off_h = slot.off - Td;
    slot.take(Tf1); P.off_u = slot.off - Tf1;
    const size_t stat = ((size_t)D.T * 4 + 255) & ~(size_t)255;   // mean1, rstd1, mean2, rstd2: 256-byte aligned each
    slot.take(4 * stat); P.off_stats = slot.off - 4 * stat;
    slot.take((size_t)D.B * D.H * D.S * 4); P.off_lse = slot.off - (size_t)D.B * D.H * D.S * 4;
    slot.take(Td); P.off_x = slot.off - Td;
    P.app_pitch = slot.total();
  }
  P.app_slots = (char*)cv.take(D.apps * P.app_pitch);
  P.du_slots = (char*)cv.take(R * Tf1); P.dh_slots = (char*)cv.take(R * Td); P.dqkv_slots = (char*)cv.take(R * 3 * Td);
  P.dys[0] = D.apps > 1 ? (char*)cv.take(R * Td) : nullptr;
  P.dys[1] = L > 1 ? (char*)cv.take(R * Td) : nullptr;
  P.t.dg = D.rope_geglu ? cv.take(Tf) : nullptr;
  P.t.dc = cv.take(Td); P.t.dout = cv.take(Td); P.t.da = cv.take(Td);
  P.t.delta = (float*)cv.take((size_t)D.B * D.H * D.S * 4);
  size_t pf = layernorm_bwd_scratch_floats(D.T, D.d);
  pf = std::max(pf, colsum_scratch_floats(wgrad_chunk(D, R) * D.T, std::max(3 * D.d, D.f1)));
  P.t.partial = (float*)cv.take(pf * 4);
  P.splitk = splitk_floats_of(D) ? (float*)cv.take(splitk_floats_of(D) * 4) : nullptr;
  return cv.total();
}

// Where application i keeps the input it was given by application i - 1 (i >= 1).
void* input_buffer_at(const BwdPlan& P, int i) { return P.app_slots + (size_t)i * P.app_pitch + P.off_x; }

// Intermediates of application i; `x` = its input.
Saved saved_at(const BwdPlan& P, const Dims& D, int i, const void* x) {
  const size_t Td = (size_t)D.T * D.d * D.es, Tf = (size_t)D.T * D.f * D.es;
  char* slot = P.app_slots + (size_t)i * P.app_pitch;
  Saved s{};
  s.x = x;
  s.a = P.a_all + i * Td; s.o = P.o_all + i * Td; s.c = P.c_all + i * Td; s.g = P.g_all + i * Tf;
  s.qkv = slot; s.h = slot + P.off_h; s.u = slot + P.off_u;
  float* stats = (float*)(slot + P.off_stats);
  const size_t stat = (((size_t)D.T * 4 + 255) & ~(size_t)255) / 4;
  s.mean1 = stats; s.rstd1 = stats + stat; s.mean2 = stats + 2 * stat; s.rstd2 = stats + 3 * stat;
  s.lse = (float*)(slot + P.off_lse);
  s.rope = P.rope;
  return s;
}

// Recompute the forward from the stage input (keeping every application's intermediates), then the reverse
// sweep.  grad_in == nullptr: the input gradient leaves int8-encoded in gin_codes / gin_scales.
swarm_status run_backward(const Dims& D, const swarm_stage_config* cfg, const swarm_block_params* params,
                          const void* x_in, const void* grad_out, void* grad_in, int8_t* gin_codes,
                          void* gin_scales, const swarm_block_grads* grad_params, const BwdPlan& P,
                          hipStream_t st, bool scales16 = false) {
  const int L = cfg->n_layers, R = cfg->n_repeat;
  const size_t Td = (size_t)D.T * D.d * D.es, Tf1 = (size_t)D.T * D.f1 * D.es;
  if (P.rope) SWARM_TRY(rope_table(P.rope, D.S, D.dh, st));
  const void* cur = x_in;
  int app = 0;
  for (int l = 0; l < L; ++l)
    for (int r = 0; r < R; ++r, ++app) {
      void* y = (app == D.apps - 1) ? nullptr : input_buffer_at(P, app + 1);   // the stage output is not needed
      SWARM_TRY(block_forward(D, params[l], saved_at(P, D, app, cur), y, cfg->ln_eps, st));
      cur = y;
    }
  // With sharing, the last application's output gradient joins the slots of its parameter set, so that the set's
  // weight gradients stay one product over all its applications: one copy of a [T,d] tensor against a second
  // read-modify-write pass over the set's fp32 gradient matrices.  Without sharing grad_out is read in place.
  const bool direct = R == 1;
  if (!direct &&
      hipMemcpyAsync(P.dys[(L - 1) & 1] + (size_t)(R - 1) * Td, grad_out, Td, hipMemcpyDeviceToDevice, st) != hipSuccess)
    return SWARM_ERR_LAUNCH;
  const int chunk = wgrad_chunk(D, R);
  for (int l = L - 1; l >= 0; --l) {
    char* base = P.dys[l & 1];
    const bool from_caller = direct && l == L - 1;
    for (int r = R - 1; r >= 0; --r) {
      app = l * R + r;
      const void* dy = from_caller ? grad_out : base + (size_t)r * Td;
      const AppGrads ag{P.du_slots + (size_t)r * Tf1, P.dh_slots + (size_t)r * Td, P.dqkv_slots + (size_t)r * 3 * Td};
      const Saved sv = saved_at(P, D, app, app == 0 ? x_in : input_buffer_at(P, app));
      if (app == 0) {
        SWARM_TRY(block_backward(D, params[l], grad_params[l], sv, P.t, ag, dy, grad_in, st,
                                 grad_in ? nullptr : gin_codes, grad_in ? nullptr : gin_scales, scales16));
      } else {
        void* dx = r > 0 ? base + (size_t)(r - 1) * Td : P.dys[(l - 1) & 1] + (size_t)(R - 1) * Td;
        SWARM_TRY(block_backward(D, params[l], grad_params[l], sv, P.t, ag, dy, dx, st));
      }
    }
    for (int r0 = 0; r0 < R; r0 += chunk) {
      const int n = std::min(chunk, R - r0);
      const void* dy = from_caller ? grad_out : base + (size_t)r0 * Td;
      const AppGrads ag{P.du_slots + (size_t)r0 * Tf1, P.dh_slots + (size_t)r0 * Td,
                        P.dqkv_slots + (size_t)r0 * 3 * Td};
      SWARM_TRY(set_weight_grads(D, grad_params[l], n, dy, ag, saved_at(P, D, l * R + r0, nullptr), P.t.partial, st));
    }
  }
  return SWARM_OK;
}

bool params_ok(const swarm_block_params* p, int L) {
  for (int l = 0; l < L; ++l) {
    const void* const* f = (const void* const*)&p[l];
    for (int i = 0; i < 12; ++i)
      if (!f[i]) return false;
  }
  return true;
}

bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

}  // namespace
}  // namespace swarm

using namespace swarm;

extern "C" size_t swarm_stage_workspace_bytes(const swarm_stage_config* cfg, int for_backward) {
  if (!valid_config(cfg)) return 0;
  const Dims D = dims_of(cfg);
  if (for_backward) {
    BwdPlan P;
    return plan_backward(D, cfg->n_layers, cfg->n_repeat, nullptr, P);
  }
  FwdPlan P;
  return plan_forward(D, nullptr, P);
}

extern "C" swarm_status swarm_stage_forward(const swarm_stage_config* cfg, const swarm_block_params* params,
                                            const void* x_in, void* x_out, void* workspace, size_t workspace_bytes,
                                            void* hip_stream) {
  if (!cfg || !params || !x_in || !x_out || !workspace) return SWARM_ERR_NULL;
  if (cfg->dtype != SWARM_F32 && cfg->dtype != SWARM_BF16) return SWARM_ERR_DTYPE;
  if (!valid_config(cfg)) return SWARM_ERR_SHAPE;
  if (!params_ok(params, cfg->n_layers)) return SWARM_ERR_NULL;
  if (x_in == x_out || !aligned16(x_in) || !aligned16(x_out) || ((uintptr_t)workspace & 255)) return SWARM_ERR_SHAPE;
  Dims D = dims_of(cfg);
  FwdPlan P;
  if (plan_forward(D, workspace, P) > workspace_bytes) return SWARM_ERR_WORKSPACE;
  D.splitk = P.splitk; D.splitk_floats = P.splitk ? splitk_floats_of(D) : 0;
  hipStream_t st = (hipStream_t)hip_stream;
  if (P.rope) SWARM_TRY(rope_table(P.rope, D.S, D.dh, st));
  const void* cur = x_in;
  int app = 0;
  for (int l = 0; l < cfg->n_layers; ++l)
    for (int r = 0; r < cfg->n_repeat; ++r, ++app) {
      void* y = (app == D.apps - 1) ? x_out : P.z[app & 1];
      P.s.x = cur;
      SWARM_TRY(block_forward(D, params[l], P.s, y, cfg->ln_eps, st, Boundary(), false));
      cur = y;
    }
  return SWARM_OK;
}

extern "C" swarm_status swarm_stage_backward(const swarm_stage_config* cfg, const swarm_block_params* params,
                                             const void* x_in, const void* grad_out, void* grad_in,
                                             const swarm_block_grads* grad_params, void* workspace,
                                             size_t workspace_bytes, void* hip_stream) {
  if (!cfg || !params || !x_in || !grad_out || !grad_in || !grad_params || !workspace) return SWARM_ERR_NULL;
  if (cfg->dtype != SWARM_F32 && cfg->dtype != SWARM_BF16) return SWARM_ERR_DTYPE;
  if (!valid_config(cfg)) return SWARM_ERR_SHAPE;
  if (!params_ok(params, cfg->n_layers) || !params_ok((const swarm_block_params*)grad_params, cfg->n_layers))
    return SWARM_ERR_NULL;
  if (grad_in == grad_out || grad_in == x_in || !aligned16(x_in) || !aligned16(grad_out) || !aligned16(grad_in) ||
      ((uintptr_t)workspace & 255))
    return SWARM_ERR_SHAPE;
  Dims D = dims_of(cfg);
  BwdPlan P;
  if (plan_backward(D, cfg->n_layers, cfg->n_repeat, workspace, P) > workspace_bytes) return SWARM_ERR_WORKSPACE;
  D.splitk = P.splitk; D.splitk_floats = P.splitk ? splitk_floats_of(D) : 0;
  return run_backward(D, cfg, params, x_in, grad_out, grad_in, nullptr, nullptr, grad_params, P,
                      (hipStream_t)hip_stream);
}

// ---------------------------------------------------------------------------------------------
// Entry points with the boundary codec fused into the stage.  Fused kernels are used for bf16 with
// d_model % 256 == 0; otherwise the same results come from the stand-alone codec kernels around the stage.
namespace swarm {
namespace {
bool fuse_codec(const Dims& D) { return D.bf16 && D.d % 256 == 0; }
}  // namespace
}  // namespace swarm

extern "C" size_t swarm_stage_coded_workspace_bytes(const swarm_stage_config* cfg, int for_backward) {
  const size_t base = swarm_stage_workspace_bytes(cfg, for_backward);
  if (!base) return 0;
  const Dims D = dims_of(cfg);
  return base + 256 + 2 * (((size_t)D.T * D.d * D.es + 255) & ~(size_t)255);   // two boundary tensors of scratch
}

namespace swarm {
namespace {

swarm_status forward_coded(const swarm_stage_config* cfg, const swarm_block_params* params, const int8_t* x_codes,
                           const void* x_scales, void* x_dec, int8_t* y_codes, void* y_scales, void* workspace,
                           size_t workspace_bytes, void* hip_stream, bool scales16) {
  if (!cfg || !params || !x_codes || !x_scales || !x_dec || !y_codes || !y_scales || !workspace) return SWARM_ERR_NULL;
  if (cfg->dtype != SWARM_F32 && cfg->dtype != SWARM_BF16) return SWARM_ERR_DTYPE;
  if (!valid_config(cfg)) return SWARM_ERR_SHAPE;
  if (!params_ok(params, cfg->n_layers)) return SWARM_ERR_NULL;
  if (!aligned16(x_dec) || !aligned16(x_codes) || !aligned16(y_codes) || ((uintptr_t)workspace & 255) ||
      (((uintptr_t)x_scales | (uintptr_t)y_scales) & (scales16 ? 1 : 3)))
    return SWARM_ERR_SHAPE;
  if (swarm_stage_coded_workspace_bytes(cfg, 0) > workspace_bytes) return SWARM_ERR_WORKSPACE;
  Dims D = dims_of(cfg);
  hipStream_t st = (hipStream_t)hip_stream;
  const size_t base = swarm_stage_workspace_bytes(cfg, 0);
  void* tmp = (char*)workspace + ((base + 255) & ~(size_t)255);
  const size_t n = (size_t)D.T * D.d;
  if (!fuse_codec(D)) {
    SWARM_TRY(codec_decode_launch(x_codes, x_scales, n, x_dec, D.bf16, st, scales16));
    SWARM_TRY(swarm_stage_forward(cfg, params, x_dec, tmp, workspace, base, hip_stream));
    return codec_encode_launch(tmp, n, y_codes, y_scales, D.bf16, st, scales16);
  }
  FwdPlan P;
  plan_forward(D, workspace, P);
  D.splitk = P.splitk; D.splitk_floats = P.splitk ? splitk_floats_of(D) : 0;
  if (P.rope) SWARM_TRY(rope_table(P.rope, D.S, D.dh, st));
  const void* cur = x_dec;
  int app = 0;
  for (int l = 0; l < cfg->n_layers; ++l)
    for (int r = 0; r < cfg->n_repeat; ++r, ++app) {
      const bool last = app == D.apps - 1;
      Boundary bd;
      bd.scales16 = scales16;
      if (app == 0) { bd.in_codes = x_codes; bd.in_scales = x_scales; }
      if (last) { bd.out_codes = y_codes; bd.out_scales = y_scales; }
      void* y = last ? nullptr : P.z[app & 1];
      P.s.x = cur;
      SWARM_TRY(block_forward(D, params[l], P.s, y, cfg->ln_eps, st, bd, false));
      cur = y;
    }
  return SWARM_OK;
}

swarm_status backward_coded(const swarm_stage_config* cfg, const swarm_block_params* params, const void* x_in,
                            const int8_t* g_codes, const void* g_scales, int8_t* gin_codes, void* gin_scales,
                            const swarm_block_grads* grad_params, void* workspace, size_t workspace_bytes,
                            void* hip_stream, bool scales16) {
  if (!cfg || !params || !x_in || !g_codes || !g_scales || !gin_codes || !gin_scales || !grad_params || !workspace)
    return SWARM_ERR_NULL;
  if (cfg->dtype != SWARM_F32 && cfg->dtype != SWARM_BF16) return SWARM_ERR_DTYPE;
  if (!valid_config(cfg)) return SWARM_ERR_SHAPE;
  if (!params_ok(params, cfg->n_layers) || !params_ok((const swarm_block_params*)grad_params, cfg->n_layers))
    return SWARM_ERR_NULL;
  if (!aligned16(x_in) || !aligned16(g_codes) || !aligned16(gin_codes) || ((uintptr_t)workspace & 255) ||
      (((uintptr_t)g_scales | (uintptr_t)gin_scales) & (scales16 ? 1 : 3)))
    return SWARM_ERR_SHAPE;
  if (swarm_stage_coded_workspace_bytes(cfg, 1) > workspace_bytes) return SWARM_ERR_WORKSPACE;
  Dims D = dims_of(cfg);
  hipStream_t st = (hipStream_t)hip_stream;
  const size_t base = swarm_stage_workspace_bytes(cfg, 1);
  void* tmp = (char*)workspace + ((base + 255) & ~(size_t)255);
  const size_t n = (size_t)D.T * D.d;
  // the output gradient has several readers (bias sums, two GEMMs, LayerNorm backward): decode it once
  SWARM_TRY(codec_decode_launch(g_codes, g_scales, n, tmp, D.bf16, st, scales16));
  if (!fuse_codec(D)) {
    void* gin = (char*)tmp + (((size_t)D.T * D.d * D.es + 255) & ~(size_t)255);
    SWARM_TRY(swarm_stage_backward(cfg, params, x_in, tmp, gin, grad_params, workspace, base, hip_stream));
    return codec_encode_launch(gin, n, gin_codes, gin_scales, D.bf16, st, scales16);
  }
  BwdPlan P;
  plan_backward(D, cfg->n_layers, cfg->n_repeat, workspace, P);
  D.splitk = P.splitk; D.splitk_floats = P.splitk ? splitk_floats_of(D) : 0;
  return run_backward(D, cfg, params, x_in, tmp, nullptr, gin_codes, gin_scales, grad_params, P, st, scales16);
}

}  // namespace
}  // namespace swarm

extern "C" swarm_status swarm_stage_forward_coded(const swarm_stage_config* cfg, const swarm_block_params* params,
                                                  const int8_t* x_codes, const float* x_scales, void* x_dec,
                                                  int8_t* y_codes, float* y_scales, void* workspace,
                                                  size_t workspace_bytes, void* hip_stream) {
  return forward_coded(cfg, params, x_codes, x_scales, x_dec, y_codes, y_scales, workspace, workspace_bytes,
                       hip_stream, false);
}

extern "C" swarm_status swarm_stage_backward_coded(const swarm_stage_config* cfg, const swarm_block_params* params,
                                                   const void* x_in, const int8_t* g_codes, const float* g_scales,
                                                   int8_t* gin_codes, float* gin_scales,
                                                   const swarm_block_grads* grad_params, void* workspace,
                                                   size_t workspace_bytes, void* hip_stream) {
  return backward_coded(cfg, params, x_in, g_codes, g_scales, gin_codes, gin_scales, grad_params, workspace,
                        workspace_bytes, hip_stream, false);
}

extern "C" swarm_status swarm_stage_forward_coded_s16(const swarm_stage_config* cfg, const swarm_block_params* params,
                                                      const int8_t* x_codes, const uint16_t* x_scales, void* x_dec,
                                                      int8_t* y_codes, uint16_t* y_scales, void* workspace,
                                                      size_t workspace_bytes, void* hip_stream) {
  return forward_coded(cfg, params, x_codes, x_scales, x_dec, y_codes, y_scales, workspace, workspace_bytes,
                       hip_stream, true);
}

extern "C" swarm_status swarm_stage_backward_coded_s16(const swarm_stage_config* cfg, const swarm_block_params* params,
                                                       const void* x_in, const int8_t* g_codes,
                                                       const uint16_t* g_scales, int8_t* gin_codes,
                                                       uint16_t* gin_scales, const swarm_block_grads* grad_params,
                                                       void* workspace, size_t workspace_bytes, void* hip_stream) {
  return backward_coded(cfg, params, x_in, g_codes, g_scales, gin_codes, gin_scales, grad_params, workspace,
                        workspace_bytes, hip_stream, true);
}
