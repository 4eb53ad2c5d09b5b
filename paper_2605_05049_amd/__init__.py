"""MI355X-native MoE expert layer (gfx950 HIP kernels behind a C ABI); thin ctypes binding.

Every function here only marshals arguments (torch tensors -> device pointers, current stream) and calls the
entry point of the same name declared in include/moe.h.  There is no CPU or eager fallback: if the shared
library is missing, calls raise.
"""
from .binding import (  # noqa: F401
    MoeError, Shape, abi_version, load_library, library_path, status_str, workspace_bytes,
    moe_route_topk, moe_route_topk_bwd, moe_permute, moe_permute_noalloc, moe_permute_bwd, moe_permute_bwd_add, moe_router_fwd,
    moe_router_bwd, moe_grouped_ffn_bwd_recompute, moe_grouped_ffn_fwd,
    moe_grouped_ffn_bwd, moe_unpermute_combine, moe_unpermute_combine_bwd, EXPORTED_SYMBOLS,
    profile_enable, profile_reset, profile_records, load_accumulate, load_imbalance, rebalance_experts,
    moe_halo_pack_remote, moe_halo_repack, moe_halo_unpack,
)
from .layer import MoeLayerBuffers, CapturedLayerStep, layer_forward, layer_backward  # noqa: F401
