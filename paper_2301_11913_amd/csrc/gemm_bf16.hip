#include "kernels.h"
namespace swarm {
swarm_status gemm_bf16(const GemmArgs& g, hipStream_t st) { return gemm_generic(g, true, st); }
}
