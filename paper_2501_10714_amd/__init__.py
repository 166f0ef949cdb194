"""MI355X-native single-GPU MoE layer hot path: thin Python binding over the C-ABI HIP library.

The binding only marshals arguments; every step runs in the library's kernels.  There is no CPU
fallback: loading fails loudly when the library has not been built.
"""
from .binding import (MoeConfig, MoeError, lib_path, load, moe_capacity, moe_combine, moe_combine_bwd,  # noqa: F401
                      moe_layer_fwd_chunked, moe_layer_bwd_chunked, MAX_CHUNKS, PipelineModel, moe_pipeline_time,
                      moe_find_pipeline_degree, moe_route_noisy, moe_route_noisy_bwd, moe_route_xmoe,
                      moe_route_xmoe_bwd, moe_route_xmoe_workspace_bytes, moe_layer_fwd_routed, moe_layer_bwd_routed,
                      moe_dispatch, moe_dispatch_bwd, moe_expert_ffn_bwd, moe_expert_ffn_fwd, moe_last_error,
                      moe_layer_bwd, moe_layer_fwd, moe_route, moe_route_static, moe_route_bwd, moe_saved_offset, moe_workspace_bytes,
                      saved_view, ACT_GELU_ERF, ACT_GELU_TANH, ACT_RELU, ACT_SWIGLU, DT_BF16, DT_F32, SAVED)
