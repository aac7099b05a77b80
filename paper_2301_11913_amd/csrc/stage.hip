#include "common.h"
extern "C" size_t swarm_stage_workspace_bytes(const swarm_stage_config*, int) { return 0; }
extern "C" swarm_status swarm_stage_forward(const swarm_stage_config*, const swarm_block_params*, const void*, void*, void*, size_t, void*) { return SWARM_ERR_SHAPE; }
extern "C" swarm_status swarm_stage_backward(const swarm_stage_config*, const swarm_block_params*, const void*, const void*, void*, const swarm_block_grads*, void*, size_t, void*) { return SWARM_ERR_SHAPE; }
