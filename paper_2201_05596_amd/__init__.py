"""MI355X-native forward pass of one Mixture-of-Experts layer (DeepSpeed-MoE,
arXiv 2201.05596, Sec. 5.4 / 4.1.1): thin Python binding over libmoe_hip.so."""
from .binding import (MOE_BF16, MOE_F32, MOE_FLAG_PACKED_WEIGHTS, MOE_FLAG_PACKED_GATE, moe_pack_gate, moe_packed_gate_bytes, moe_pack_weights, moe_packed_weights_bytes, ENTRY_POINTS, LIB_PATH, MoeError, MoeShape, alloc_workspace, load_library,
                      make_shape, moe_combine, moe_dispatch, moe_expert_ffn, moe_expert_ffn_slice, moe_expert_ffn_slice_reduce, moe_gate, moe_gate_noalloc, moe_gate_noalloc_bytes,
                      moe_gate_noalloc_max_bytes, moe_layer_forward, moe_decode_block_forward, moe_decode_block_workspace_bytes, MoeBlockShape,
                      moe_version, moe_workspace_bytes, moe_profile_enable, moe_profile_select, moe_profile_stride, moe_profile_calls,
                      moe_profile_stage_names, moe_profile_elapsed)
from .layer import MoELayer

__all__ = ["MOE_BF16", "MOE_F32", "MOE_FLAG_PACKED_WEIGHTS", "MOE_FLAG_PACKED_GATE", "moe_pack_gate", "moe_packed_gate_bytes", "moe_pack_weights", "moe_packed_weights_bytes", "ENTRY_POINTS", "LIB_PATH", "MoeError", "MoeShape", "alloc_workspace",
           "load_library", "make_shape", "moe_combine", "moe_dispatch", "moe_expert_ffn", "moe_expert_ffn_slice", "moe_expert_ffn_slice_reduce", "moe_gate", "moe_gate_noalloc", "moe_gate_noalloc_bytes", "moe_gate_noalloc_max_bytes",
           "moe_layer_forward", "moe_decode_block_forward", "moe_decode_block_workspace_bytes", "MoeBlockShape", "moe_version", "moe_workspace_bytes", "MoELayer", "moe_profile_enable", "moe_profile_select", "moe_profile_stride",
           "moe_profile_calls", "moe_profile_stage_names", "moe_profile_elapsed"]
