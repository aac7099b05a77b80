/*
 * swarm_boundary.h - C ABI of the compression-aware stage-boundary layers (MI355X, gfx950).
 *
 * The appendix "Compression-Aware Architectures" (paragraphs "Bottleneck layers" and "Maxout compression") puts a
 * learned compression at every point where activations cross from one pipeline stage to the next:
 *     Bottleneck = LayerNorm(LayerNorm(MLP(x)) w_c) w_d          Maxout = LayerNorm(maxout_k(LayerNorm(MLP(x)))) w_d
 * with w_c on the sending stage and w_d on the receiving one.  This header is that layer cut at the network:
 *     sender   ("compress"):    z = LayerNorm(y; ln_g, ln_b) w_c^T               bottleneck, w_c [c, m]
 *                               z = maxout_k(LayerNorm(y; ln_g, ln_b)), k = m/c   maxout (no matrix)
 *     receiver ("decompress"):  x = LayerNorm(z; ln_g, ln_b) w_d^T               w_d [m, c]
 * y [T, m] is the output of the sender's last Transformer block, z [T, c] is what travels (it may additionally go
 * through swarm_codec_encode / swarm_codec_decode), x [T, m] is the input of the receiver's first block.
 * maxout_k(a)[t, j] = max_{i<k} a[t, j*k + i]; its gradient goes to the first maximal feature of the window.
 * LayerNorm: biased variance, eps inside the square root, learned gain and bias; the linear maps have no bias.
 *
 * The backward calls follow the stage's checkpointing rule (Section 3.2): they get the layer INPUT and the gradient
 * of its output, recompute what they need, return the gradient of the input and ADD the parameter gradients
 * (fp32) to the caller's buffers.
 *
 * General rules: those of swarm_stage.h (device pointers owned by the caller, host structs read during the call,
 * nothing allocated or retained, work enqueued on `hip_stream`, host-visible errors returned before any launch,
 * bitwise reproducible).
 */
#ifndef SWARM_BOUNDARY_H
#define SWARM_BOUNDARY_H

#include "swarm_stage.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { SWARM_COMPRESS_BOTTLENECK = 0, SWARM_COMPRESS_MAXOUT = 1 } swarm_compress_kind;

/* Constraints: d_model % 64 == 0, d_model <= 8192; d_comp % 32 == 0, 32 <= d_comp <= d_model; maxout: d_model %
 * d_comp == 0 (k = d_model / d_comp); tokens >= 1. */
typedef struct {
  int32_t d_model;   /* m                                                  */
  int32_t d_comp;    /* c: width of z                                      */
  int32_t kind;      /* swarm_compress_kind                                */
  int32_t tokens;    /* T = microbatch * sequence length                   */
  int32_t dtype;     /* swarm_dtype of y, z, x, their gradients, parameters */
  float   ln_eps;
} swarm_boundary_config;

typedef struct { const void *ln_g, *ln_b; /* [m] */ const void *w_c; /* [c, m]; NULL for maxout */ } swarm_compress_params;
typedef struct { float *ln_g, *ln_b, *w_c; } swarm_compress_grads;       /* same shapes, fp32, ADDED to */
typedef struct { const void *ln_g, *ln_b; /* [c] */ const void *w_d; /* [m, c] */ } swarm_decompress_params;
typedef struct { float *ln_g, *ln_b, *w_d; } swarm_decompress_grads;

/* Bytes of 256-byte aligned device workspace for the call named by (decompress != 0, for_backward != 0);
 * 0 if the config is invalid. */
size_t swarm_boundary_workspace_bytes(const swarm_boundary_config *cfg, int decompress, int for_backward);

/* Sender, forward: y [T, m] -> z [T, c] (overwritten; must not alias y). */
swarm_status swarm_compress_forward(const swarm_boundary_config *cfg, const swarm_compress_params *params,
                                    const void *y, void *z, void *workspace, size_t workspace_bytes, void *hip_stream);
/* Sender, backward: y, dz [T, c] -> dy [T, m] (overwritten; must not alias y or dz); grads are added to. */
swarm_status swarm_compress_backward(const swarm_boundary_config *cfg, const swarm_compress_params *params,
                                     const void *y, const void *dz, void *dy, const swarm_compress_grads *grads,
                                     void *workspace, size_t workspace_bytes, void *hip_stream);
/* Receiver, forward: z [T, c] -> x [T, m] (overwritten; must not alias z). */
swarm_status swarm_decompress_forward(const swarm_boundary_config *cfg, const swarm_decompress_params *params,
                                      const void *z, void *x, void *workspace, size_t workspace_bytes,
                                      void *hip_stream);
/* Receiver, backward: z, dx [T, m] -> dz [T, c] (overwritten; must not alias z or dx); grads are added to. */
swarm_status swarm_decompress_backward(const swarm_boundary_config *cfg, const swarm_decompress_params *params,
                                       const void *z, const void *dx, void *dz, const swarm_decompress_grads *grads,
                                       void *workspace, size_t workspace_bytes, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* SWARM_BOUNDARY_H */
