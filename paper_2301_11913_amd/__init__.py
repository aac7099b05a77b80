"""MI355X-native pipeline-stage library for SWARM parallelism: Python binding.

The compute lives in libswarm_stage.so (hand-written HIP for gfx950, C ABI in
include/swarm_stage.h).  This package only marshals arguments; PyTorch supplies
device memory and streams.  There is no CPU fallback: a missing library raises.
"""
from .binding import (  # noqa: F401
    SWARM_F32, SWARM_BF16, SWARM_BLOCK_GELU, SWARM_BLOCK_ROTARY_GEGLU, SwarmError, StageConfig, lib_path, load_library,
    hooks_lib_path, load_hooks_library, using_hooks_library,
    swarm_stage_workspace_bytes, swarm_stage_forward, swarm_stage_backward,
    swarm_codec_encode, swarm_codec_decode, swarm_status_string,
    swarm_stage_coded_workspace_bytes, swarm_stage_forward_coded, swarm_stage_backward_coded,
    PARAM_FIELDS, EXPORTED_SYMBOLS,
    SWARM_COMPRESS_BOTTLENECK, SWARM_COMPRESS_MAXOUT, BoundaryConfig,
    swarm_boundary_workspace_bytes, swarm_compress_forward, swarm_compress_backward,
    swarm_decompress_forward, swarm_decompress_backward,
    HeadConfig, swarm_embedding_forward, swarm_embedding_backward, swarm_head_workspace_bytes,
    swarm_head_loss, swarm_head_loss_backward,
    swarm_lamb_workspace_bytes, swarm_lamb_step, swarm_lamb_step_static, SWARM_LAMB_STATIC_MAX_ELEMS,
    swarm_codec_encode_s16, swarm_codec_decode_s16,
)
