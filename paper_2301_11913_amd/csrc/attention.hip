// Attention dispatch: MFMA flash kernels for bf16, direct kernels otherwise.
#include "kernels.h"

namespace swarm {

swarm_status attention_fwd_naive(const void*, void*, float*, int, int, int, int, bool, hipStream_t);
swarm_status attention_bwd_naive(const void*, const void*, const void*, const float*, float*, void*, int, int, int,
                                 int, bool, hipStream_t);

swarm_status attention_fwd_mfma(const void*, void*, float*, int, int, int, int, hipStream_t);

swarm_status attention_fwd(const void* qkv, void* o, float* lse, int B, int S, int H, int dh, bool bf16,
                           hipStream_t st) {
  if (bf16 && (dh == 64 || dh == 128)) return attention_fwd_mfma(qkv, o, lse, B, S, H, dh, st);
  return attention_fwd_naive(qkv, o, lse, B, S, H, dh, bf16, st);
}

swarm_status attention_bwd_mfma(const void*, const void*, const void*, const float*, float*, void*, int, int, int,
                                int, hipStream_t);

swarm_status attention_bwd(const void* qkv, const void* o, const void* dout, const float* lse, float* delta,
                           void* dqkv, int B, int S, int H, int dh, bool bf16, hipStream_t st) {
  if (bf16 && (dh == 64 || dh == 128)) return attention_bwd_mfma(qkv, o, dout, lse, delta, dqkv, B, S, H, dh, st);
  return attention_bwd_naive(qkv, o, dout, lse, delta, dqkv, B, S, H, dh, bf16, st);
}

}  // namespace swarm
