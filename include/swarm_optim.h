/*
 * swarm_optim.h - C ABI of the optimiser step (MI355X, gfx950).
 *
 * Once the peers of a stage have averaged their accumulated gradients (Section 3.2), each applies the optimiser;
 * the large-scale run uses LAMB with learning rate 1e-3 and beta2 = 0.95 (appendix "Additional Details for
 * Section 4.3").  One call updates ONE parameter tensor (LAMB's trust ratio is per tensor):
 *     g  = grad_scale * grad
 *     m <- beta1 m + (1 - beta1) g                 v <- beta2 v + (1 - beta2) g^2
 *     r  = (m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) + eps)
 *     u  = r + weight_decay * w
 *     w <- w - lr * (||w|| / ||u||) * u            (ratio 1 when either norm is zero)
 * All state is fp32 on the device: `master` (the weights), `m`, `v`; `grad` is the fp32 gradient buffer that the
 * stage calls accumulate into (read only here; the caller zeroes it for the next global batch).  When `param` is
 * not NULL the updated weights are also written there in `dtype` (the bf16 copy the stage kernels read).
 * The norms are reduced in a fixed order (no atomics): results are bitwise reproducible.
 *
 * General rules: those of swarm_stage.h.
 */
#ifndef SWARM_OPTIM_H
#define SWARM_OPTIM_H

#include "swarm_stage.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
  float lr, beta1, beta2, eps, weight_decay;
  float grad_scale;   /* e.g. 1 / (number of microbatches accumulated) */
  int32_t step;       /* t >= 1 */
} swarm_lamb_config;

/* Bytes of 256-byte aligned device workspace for a tensor of n elements (the update direction u and the partial
 * sums of the two norms). */
size_t swarm_lamb_workspace_bytes(size_t n_elems);

/* n_elems >= 1; master, grad, m, v: fp32 [n_elems]; param: `dtype` [n_elems] or NULL.  master, m, v (and param)
 * are updated in place.  If trust_ratio != NULL the ratio used is written there (device fp32 scalar). */
swarm_status swarm_lamb_step(const swarm_lamb_config *cfg, size_t n_elems, float *master, void *param, int32_t dtype,
                             const float *grad, float *m, float *v, float *trust_ratio, void *workspace,
                             size_t workspace_bytes, void *hip_stream);

/* swarm_lamb_step for callers that cannot allocate device memory or carry a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the same three kernels with their scratch (update
 * direction, partial sums of the norms, ratio) in a static device array inside the library, 64 MiB + 33 KiB per GPU,
 * held from the library's load until the process ends.  n_elems <= SWARM_LAMB_STATIC_MAX_ELEMS (one 4096 x 4096
 * matrix), SWARM_ERR_WORKSPACE beyond; everything else as swarm_lamb_step, and the results are bit-identical to it.
 * The call allocates and frees nothing.  All calls on one GPU share that GPU's array: calls that may overlap there
 * (different streams, different threads) race; calls on one stream are ordered and safe.  Nothing has to be
 * cleared between calls: every scratch word a call reads has been written by that call first. */
#define SWARM_LAMB_STATIC_MAX_ELEMS ((size_t)1 << 24)
swarm_status swarm_lamb_step_static(const swarm_lamb_config *cfg, size_t n_elems, float *master, void *param,
                                    int32_t dtype, const float *grad, float *m, float *v, float *trust_ratio,
                                    void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* SWARM_OPTIM_H */
