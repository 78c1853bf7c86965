"""MI355X (gfx950) MoE-layer library: Python binding of the C ABI in include/moe.h.

The five calls of the layer -- moe_route, moe_permute, moe_expert_ffn,
moe_combine and the fused moe_layer -- plus the page packer, the page
streamer and the multi-layer weight-paging pipeline.  All compute runs in the HIP library (libmoe_hip.so, built in-tree by
``paper_2411_11217_amd.build``); there is no CPU or PyTorch fallback.
"""
from .binding import (  # noqa: F401
    DTYPE_BF16, DTYPE_F32, EXPORTED_SYMBOLS, LinearShape, MAX_EXPERTS, MoEError, MoEShape, Pipeline, STATIC_SCRATCH_BYTES, Streamer, Workspace,
    get_option, library_path, linear_pack, linear_pages_required, make_linear_shape, make_shape, moe_add_rmsnorm,
    moe_cast_bf16, moe_linear, moe_post_attention, moe_pre_attention, post_attention_workspace_bytes, moe_combine, moe_expert_ffn, moe_expert_ffn_streamed, moe_layer,
    moe_layer_static, moe_layer_streamed, moe_permute, moe_route, pack_weights, page_table_validate, pages_required, pipeline_pool_pages, probe_stream_read, profile_read, set_option,
    tile_bytes, unpack_weights, validate_shape, workspace_layout,
)
from .paged import PagedWeights  # noqa: F401
