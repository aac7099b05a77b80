/*
 * swarm_head.h - C ABI of the first- and last-stage extras of the language model (MI355X, gfx950).
 *
 * The first-stage embedding layer and the last-stage language-modelling head of the Section 4.3 model (the
 * appendix "Detailed Performance Comparison" describes a last stage that holds only the vocabulary projection).
 * The paper prints no formulas for them; the plain definitions are used:
 *     embedding:    x[t, :] = table[token[t], :]
 *     head + loss:  n = LayerNorm(x; ln_g, ln_b);  logits[t, v] = n[t, :] . w_vocab[v, :]  (no bias);
 *                   loss = mean over the T tokens of ( logsumexp_{v < vocab} logits[t, v] - logits[t, target[t]] ).
 * The weight matrices have `vocab_rows` >= vocab rows (a vocabulary is usually padded to a tile multiple: 50257 ->
 * 50432); rows >= vocab take no part in the loss and their gradient rows are left untouched.
 *
 * General rules: those of swarm_stage.h (device pointers owned by the caller, host structs read during the call,
 * nothing allocated or retained, work enqueued on `hip_stream`, host-visible errors returned before any launch,
 * bitwise reproducible: no float atomics, repeated token ids are summed in position order).
 * Token ids and targets are int32 device arrays with values in [0, vocab); the library cannot check device data: an
 * id outside that range is never used as an address (such a token embeds to zeros / contributes only its
 * log-sum-exp), but the result is then not meaningful.
 */
#ifndef SWARM_HEAD_H
#define SWARM_HEAD_H

#include "swarm_stage.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Embedding lookup.  tokens [T]; table [vocab_rows, d] of `dtype`; x [T, d] of `dtype` (overwritten).
 * d % 8 == 0, 1 <= T. */
swarm_status swarm_embedding_forward(const int32_t *tokens, const void *table, int32_t dtype, int32_t n_tokens,
                                     int32_t vocab, int32_t d_model, void *x, void *hip_stream);

/* Embedding gradient.  grad_table [vocab_rows, d] fp32 += scatter of dx [T, d] by token id; the rows of a repeated
 * id are added in position order by the workgroup of its first occurrence.  The duplicate search is quadratic in T:
 * T <= 65536 (SWARM_ERR_SHAPE beyond). */
swarm_status swarm_embedding_backward(const int32_t *tokens, const void *dx, int32_t dtype, int32_t n_tokens,
                                      int32_t vocab, int32_t d_model, float *grad_table, void *hip_stream);

/* Constraints: d_model % 64 == 0, d_model <= 8192; 1 <= vocab <= vocab_rows; vocab_rows % 8 == 0 (the MFMA path
 * wants vocab_rows % 256 == 0 and tokens % 128 == 0, other shapes run on slower kernels); tokens >= 1. */
typedef struct {
  int32_t d_model;
  int32_t vocab;        /* V: real tokens                              */
  int32_t vocab_rows;   /* rows of w_vocab and of its gradient          */
  int32_t tokens;       /* T = microbatch * sequence length             */
  int32_t dtype;        /* swarm_dtype of x, dx and the parameters      */
  float   ln_eps;
} swarm_head_config;

typedef struct { const void *ln_g, *ln_b; /* [d] */ const void *w_vocab; /* [vocab_rows, d] */ } swarm_head_params;
typedef struct { float *ln_g, *ln_b, *w_vocab; } swarm_head_grads;   /* same shapes, fp32, ADDED to */

/* Bytes of 256-byte aligned device workspace (for_backward != 0: swarm_head_loss_backward); 0 if invalid. */
size_t swarm_head_workspace_bytes(const swarm_head_config *cfg, int for_backward);

/* Loss only (evaluation).  x [T, d], targets [T] -> *loss (device fp32 scalar, mean over tokens) and, when
 * token_loss != NULL, the T per-token losses (device fp32). */
swarm_status swarm_head_loss(const swarm_head_config *cfg, const swarm_head_params *params, const void *x,
                             const int32_t *targets, float *loss, float *token_loss, void *workspace,
                             size_t workspace_bytes, void *hip_stream);

/* Loss and its backward in one call (what the last stage does with every microbatch): additionally dx [T, d]
 * (gradient of the mean loss w.r.t. x; overwritten; must not alias x) and grads += parameter gradients. */
swarm_status swarm_head_loss_backward(const swarm_head_config *cfg, const swarm_head_params *params, const void *x,
                                      const int32_t *targets, float *loss, float *token_loss, void *dx,
                                      const swarm_head_grads *grads, void *workspace, size_t workspace_bytes,
                                      void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* SWARM_HEAD_H */
