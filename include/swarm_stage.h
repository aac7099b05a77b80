/*
 * swarm_stage.h - C ABI of the MI355X (gfx950) pipeline-stage library.
 *
 * The library does what ONE peer of ONE SWARM pipeline stage does to ONE
 * microbatch (paper Section 3.2 "SWARM parallelism"; Section 2.1 "Pipeline
 * parallelism"): forward through the stage's Transformer blocks, backward
 * with recomputation of the forward (activation checkpointing, Section 3.2)
 * and accumulation of parameter gradients, and the 8-bit blockwise codec of
 * the tensors that cross stage boundaries (appendix "Compression-Aware
 * Architectures", paragraph "Quantized activations").
 *
 * General rules for every call:
 *   - every tensor pointer is a DEVICE pointer owned by the caller; the config
 *     and the parameter/gradient structs are HOST structs that are read during
 *     the call and never retained;
 *   - the library allocates nothing, keeps no state between calls and never
 *     frees or keeps a pointer; scratch memory comes in as `workspace`;
 *   - work is enqueued on `hip_stream` (a hipStream_t cast to void*, NULL = the
 *     default stream) and the call returns without synchronising;
 *   - errors that the host can see (null pointer, unsupported shape, small
 *     workspace) return a negative status BEFORE anything is launched and leave
 *     all outputs untouched; a failed launch returns SWARM_ERR_LAUNCH;
 *   - results are bitwise reproducible from call to call (no float atomics); which
 *     kernels run depends on the shapes, so the same rows inside a microbatch of
 *     another size agree to the rounding of the dtype, not bit for bit;
 *   - all matrices are row-major with the last index contiguous;
 *   - a call only enqueues kernels and device-to-device copies, so it may be captured into a HIP graph and
 *     replayed, once one call with the same shapes has run outside a capture on that device (the first launch of
 *     a kernel on a device sets its LDS size, which a capture does not record).
 */
#ifndef SWARM_STAGE_H
#define SWARM_STAGE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SWARM_OK = 0,
  SWARM_ERR_NULL = -1,       /* a required pointer is NULL                    */
  SWARM_ERR_SHAPE = -2,      /* a size or combination of sizes is unsupported */
  SWARM_ERR_DTYPE = -3,      /* unknown dtype                                 */
  SWARM_ERR_WORKSPACE = -4,  /* workspace smaller than *_workspace_bytes()    */
  SWARM_ERR_LAUNCH = -5      /* the HIP runtime refused a launch              */
} swarm_status;

typedef enum { SWARM_F32 = 0, SWARM_BF16 = 1 } swarm_dtype;

/* Which Transformer block the stage applies.
 *   SWARM_BLOCK_GELU         : the layer of the appendix "Additional Details for Section 4.1".
 *   SWARM_BLOCK_ROTARY_GEGLU : the layer of the large-scale model (appendix "Additional Details for
 *     Section 4.3": the standard layer with rotary position embeddings and GeGLU activations). */
typedef enum { SWARM_BLOCK_GELU = 0, SWARM_BLOCK_ROTARY_GEGLU = 1 } swarm_block_kind;

/* Shape of a stage.  Constraints: d_model % n_heads == 0; d_model / n_heads is 64
 * or 128; d_model % 64 == 0; d_ffn % 64 == 0; all counts >= 1; seq >= 1.
 * The stage applies parameter set 0 n_repeat times, then set 1 n_repeat times,
 * ... (layer sharing, Sections 2.3 and 4.3: n_layers = 1, n_repeat = R). */
typedef struct {
  int32_t d_model, n_heads, d_ffn;
  int32_t n_layers;          /* L distinct parameter sets in params[]              */
  int32_t n_repeat;          /* R consecutive applications of each parameter set   */
  int32_t batch, seq;        /* microbatch B, sequence length S                    */
  int32_t dtype;             /* swarm_dtype of x, grads w.r.t. x and parameters    */
  float   ln_eps;            /* LayerNorm epsilon, inside the square root          */
  int32_t block_kind;        /* swarm_block_kind                                   */
} swarm_stage_config;

/* One pre-LayerNorm Transformer block (the layer of the appendix "Additional
 * Details for Section 4.1": d_model, d_FFN, heads).  For a token row x:
 *   a = LN(x; ln1_g, ln1_b);  q|k|v = a w_qkv^T + b_qkv;
 *   o = per-head causal softmax(q k^T / sqrt(d_head)) v;  h = x + o w_o^T + b_o;
 *   c = LN(h; ln2_g, ln2_b);  y = h + gelu(c w_1^T + b_1) w_2^T + b_2   (erf GeLU).
 * Weights are [out, in]; rows 0..d-1 of w_qkv produce q, d..2d-1 k, 2d..3d-1 v;
 * head h owns columns h*d_head .. (h+1)*d_head-1 of q, k, v and o.
 * With SWARM_BLOCK_ROTARY_GEGLU two steps change:
 *   - before the softmax, the pairs (t[2i], t[2i+1]), i < d_head/2, of every head of q and of k at sequence
 *     position pos (0-based, restarting in every sequence of the microbatch) are rotated by the angle
 *     pos * 10000^(-2i/d_head):  t[2i]' = t[2i] cos - t[2i+1] sin,  t[2i+1]' = t[2i] sin + t[2i+1] cos;
 *   - w_1 is [2f, d] and b_1 [2f] (rows 0..f-1 = gate, f..2f-1 = up):  u = c w_1^T + b_1,
 *     y = h + (gelu(u[:f]) * u[f:]) w_2^T + b_2.
 * Element type = config.dtype. */
typedef struct {
  const void *ln1_g, *ln1_b;   /* [d]           */
  const void *w_qkv, *b_qkv;   /* [3d, d], [3d] */
  const void *w_o,   *b_o;     /* [d, d],  [d]  */
  const void *ln2_g, *ln2_b;   /* [d]           */
  const void *w_1,   *b_1;     /* [f, d],  [f]   ([2f, d], [2f] for the GeGLU block) */
  const void *w_2,   *b_2;     /* [d, f],  [d]  */
} swarm_block_params;

/* Gradients of one parameter set: same shapes, always fp32, ACCUMULATED into. */
typedef struct {
  float *ln1_g, *ln1_b, *w_qkv, *b_qkv, *w_o, *b_o, *ln2_g, *ln2_b, *w_1, *b_1, *w_2, *b_2;
} swarm_block_grads;

/* Bytes of device workspace the forward (for_backward = 0) or backward
 * (for_backward != 0) call needs for this config; 0 if the config is invalid.
 * The workspace must be 256-byte aligned. */
size_t swarm_stage_workspace_bytes(const swarm_stage_config *cfg, int for_backward);

/* Stage forward (Section 3.2: a peer applies its layers to the inputs received
 * from the previous stage).  x_in [B,S,d] -> x_out [B,S,d], both of cfg->dtype;
 * params[L] host array.  x_out is overwritten and must not alias x_in. */
swarm_status swarm_stage_forward(const swarm_stage_config *cfg, const swarm_block_params *params,
                                 const void *x_in, void *x_out,
                                 void *workspace, size_t workspace_bytes, void *hip_stream);

/* Stage backward (Section 3.2: a peer receives the gradient w.r.t. its outputs,
 * computes the gradient w.r.t. its inputs and accumulates the gradients of its
 * parameters; with activation checkpointing only x_in was kept, so the forward
 * is recomputed here).  grad_out [B,S,d] -> grad_in [B,S,d] (overwritten, must
 * not alias grad_out or x_in); grad_params[L] host array of fp32 device buffers
 * that are ADDED to (the caller zeroes them at the start of a global batch);
 * a shared parameter set receives the sum over its n_repeat applications. */
swarm_status swarm_stage_backward(const swarm_stage_config *cfg, const swarm_block_params *params,
                                  const void *x_in, const void *grad_out, void *grad_in,
                                  const swarm_block_grads *grad_params,
                                  void *workspace, size_t workspace_bytes, void *hip_stream);

/* Codec encode ("Quantized activations": dynamic 8-bit quantisation with
 * blockwise scaling).  tensor: n_elems values of `dtype`, flattened.  Per block of
 * `block` consecutive elements (the last may be short), in IEEE fp32:
 *   scale = max|x| / 127;  code = scale == 0 ? 0 : clamp(rint(x / scale), -127, 127)
 * with rint = round-half-to-even.  codes [n_elems] int8, scales [ceil(n/block)] fp32.
 * block must be 64.  n_elems == 0 is a no-op that returns SWARM_OK. */
swarm_status swarm_codec_encode(const void *tensor, int32_t dtype, size_t n_elems, int32_t block,
                                int8_t *codes, float *scales, void *hip_stream);

/* Codec decode: tensor[i] = (float)codes[i] * scales[i / block], rounded to
 * `dtype` (bf16: nearest-even).  Same constraints as encode. */
swarm_status swarm_codec_decode(const int8_t *codes, const float *scales, size_t n_elems, int32_t block,
                                void *tensor, int32_t dtype, void *hip_stream);

/* The same codec with 16-bit block scales (1.03125 instead of 1.0625 bytes per element; the paragraph puts the
 * saving against 16-bit tensors at about a factor 2): scale = bf16(max|x| / 127), nearest-even, stored as its bit pattern, and the
 * codes divide by that ROUNDED scale: code = scale == 0 ? 0 : clamp(rint(x / scale), -127, 127).  The rounding
 * moves the scale by at most 2^-8 relative, so the largest element still gets +-127 and every element's round-trip
 * error stays within half a step; a block whose scale rounds to zero (max|x| < 2^-127) is encoded as zeros.
 * scales [ceil(n/block)] uint16, 2-byte aligned; everything else as in swarm_codec_encode / swarm_codec_decode.
 * The fused stage entry points below exist for both scale widths. */
swarm_status swarm_codec_encode_s16(const void *tensor, int32_t dtype, size_t n_elems, int32_t block,
                                    int8_t *codes, uint16_t *scales, void *hip_stream);
swarm_status swarm_codec_decode_s16(const int8_t *codes, const uint16_t *scales, size_t n_elems, int32_t block,
                                    void *tensor, int32_t dtype, void *hip_stream);

/* The same two stage calls with the 8-bit codec of the "Quantized activations" paragraph fused into the
 * stage boundary: a peer receives int8-compressed activations / output gradients and sends int8-compressed
 * outputs / input gradients, so the boundary tensors need not be materialised twice.  Results are
 * bit-identical to swarm_codec_decode -> swarm_stage_forward / swarm_stage_backward -> swarm_codec_encode
 * (codec block 64; codes int8 [B*S*d], scales fp32 [B*S*d/64]).
 *   forward_coded : x_codes/x_scales = encoded stage input; x_dec [B,S,d] receives the decoded input (the
 *                   caller keeps it as x_in of the backward call); y_codes/y_scales = encoded stage output.
 *   backward_coded: x_in = decoded stage input; g_codes/g_scales = encoded grad_out;
 *                   gin_codes/gin_scales = encoded grad_in; grad_params are accumulated into as usual.
 * Workspace: swarm_stage_coded_workspace_bytes(). */
size_t swarm_stage_coded_workspace_bytes(const swarm_stage_config *cfg, int for_backward);
swarm_status swarm_stage_forward_coded(const swarm_stage_config *cfg, const swarm_block_params *params,
                                       const int8_t *x_codes, const float *x_scales, void *x_dec,
                                       int8_t *y_codes, float *y_scales,
                                       void *workspace, size_t workspace_bytes, void *hip_stream);
swarm_status swarm_stage_backward_coded(const swarm_stage_config *cfg, const swarm_block_params *params,
                                        const void *x_in, const int8_t *g_codes, const float *g_scales,
                                        int8_t *gin_codes, float *gin_scales,
                                        const swarm_block_grads *grad_params,
                                        void *workspace, size_t workspace_bytes, void *hip_stream);

/* The two fused calls with 16-bit block scales on all four boundary tensors: bit-identical to
 * swarm_codec_decode_s16 -> swarm_stage_forward / swarm_stage_backward -> swarm_codec_encode_s16.  scales are
 * uint16 [B*S*d/64] (bf16 bit patterns, 2-byte aligned); everything else as above, same workspace. */
swarm_status swarm_stage_forward_coded_s16(const swarm_stage_config *cfg, const swarm_block_params *params,
                                           const int8_t *x_codes, const uint16_t *x_scales, void *x_dec,
                                           int8_t *y_codes, uint16_t *y_scales,
                                           void *workspace, size_t workspace_bytes, void *hip_stream);
swarm_status swarm_stage_backward_coded_s16(const swarm_stage_config *cfg, const swarm_block_params *params,
                                            const void *x_in, const int8_t *g_codes, const uint16_t *g_scales,
                                            int8_t *gin_codes, uint16_t *gin_scales,
                                            const swarm_block_grads *grad_params,
                                            void *workspace, size_t workspace_bytes, void *hip_stream);

/* Static, human-readable name of a status code. */
const char *swarm_status_string(swarm_status status);

#ifdef __cplusplus
}
#endif
#endif /* SWARM_STAGE_H */
