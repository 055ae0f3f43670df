"""MI355X (gfx950) MoE-layer forward: routed experts invoked as stateless expert blocks.

The compute lives in ``libmoe_hip.so`` (hand-written HIP kernels behind the C ABI declared in
``include/moe.h``).  This package is only the ctypes binding: it marshals torch tensors (device
memory and the current stream) into those calls.  There is no CPU or PyTorch fallback: if the
library is missing or no GPU is present, the calls raise.
"""
from .binding import (MoeError, build_id, lib_path, load, moe_combine, moe_combine_parts, moe_fused_shared_sets,
                      moe_expert_group_forward_fused, moe_expert_group_forward, moe_expert_group_forward_gather,
                      moe_expert_list_forward, balanced_blocks,
                      moe_layer_forward,
                      moe_permute, moe_permute_static, moe_residual_norm, moe_route, moe_route_segments, segment_offsets, moe_shared_forward, moe_stack_forward,
                      moe_workspace_bytes, moe_probe_mfma, moe_tile_clock_buffer, LayerBuffers)
from .residency import ExpertResidency

__all__ = ["MoeError", "build_id", "lib_path", "load", "moe_route", "moe_route_segments", "segment_offsets", "moe_permute", "moe_permute_static", "moe_expert_group_forward",
           "moe_expert_group_forward_gather", "moe_expert_list_forward", "balanced_blocks",
           "moe_shared_forward", "moe_combine", "moe_combine_parts", "moe_fused_shared_sets", "moe_expert_group_forward_fused", "moe_workspace_bytes", "moe_layer_forward", "LayerBuffers",
           "moe_residual_norm", "moe_stack_forward", "moe_probe_mfma", "moe_tile_clock_buffer", "ExpertResidency"]
