"""MI355X-native MoE layer forward with a per-layer number of active experts (HIP kernels behind a C ABI)."""
from .binding import (EXPORTS, LEXI_BF16, LEXI_F32, LIB_PATH, SHARED_NONE, SHARED_SIGMOID, SHARED_UNGATED, Layer,
                      LexiError, RoutingOut, STAGE_NAMES, StageEvents, alloc_workspace, lexi_moe_layer_forward, lexi_pack_weights, lexi_moe_stack_forward,
                      lexi_moe_workspace_bytes, strerror, version)

__all__ = ["EXPORTS", "LEXI_BF16", "LEXI_F32", "LIB_PATH", "SHARED_NONE", "SHARED_SIGMOID", "SHARED_UNGATED", "Layer",
           "LexiError", "RoutingOut", "STAGE_NAMES", "StageEvents", "alloc_workspace", "lexi_moe_layer_forward", "lexi_pack_weights", "lexi_moe_stack_forward",
           "lexi_moe_workspace_bytes", "strerror", "version"]
