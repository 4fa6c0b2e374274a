"""MI355X-native MoE layer forward (route, permute, fused gate+up / down grouped GEMM, combine).

The package is a thin ctypes binding over the C ABI declared in include/moe.h; every step of
the path runs in the HIP library.  There is no CPU fallback: calling an entry point without
the built library raises.
"""
from .binding import (  # noqa: F401
    FLAG_FUSE_COMBINE,
    GATE_SIGMOID_NORM,
    GATE_SOFTMAX,
    GATE_SOFTMAX_RENORM,
    MoEConfig,
    MoEError,
    WorkspaceLayout,
    forward_workspace_layout,
    forward_workspace_size,
    ffn_kernel_name,
    ffn_workspace_size,
    lib,
    library_path,
    max_blocks,
    moe_block_schedule,
    moe_combine,
    moe_forward,
    moe_forward_staged,
    moe_grouped_ffn,
    moe_pack_weights,
    packed_weights_size,
    moe_permute,
    moe_permute_static,
    moe_route,
    permute_workspace_size,
    route_workspace_size,
    tile_m,
    workspace_size,
)
