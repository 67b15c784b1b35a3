"""MI355X-native MoE layer forward with a per-layer number of active experts (HIP kernels behind a C ABI).

The API lives in `binding` and needs the built library.  Importing the package never builds anything and never
falls back to another implementation: if liblexi_moe.so is missing or stale, every API name raises ImportError on
first use (so `python -m paper_2509_02753_amd.build` can still run to create it).
"""
_API = ["EXPORTS", "LEXI_BF16", "LEXI_F32", "LIB_PATH", "SHARED_NONE", "SHARED_SIGMOID", "SHARED_UNGATED", "Layer",
        "LexiError", "RoutingOut", "lexi_allocate_topk", "STAGE_NAMES", "StageEvents", "alloc_workspace", "lexi_moe_layer_forward", "lexi_moe_layer_forward_static",
        "lexi_pack_weights", "lexi_moe_profile_layer", "lexi_moe_stack_forward", "lexi_moe_workspace_bytes", "lexi_probe_hbm_read", "lexi_moe_down_plan",
        "lexi_probe_mfma_bf16", "strerror", "version"]
__all__ = list(_API)

try:
    from . import binding as _binding
    _load_error = None
except (ImportError, AttributeError, OSError) as exc:   # library missing, or built from older sources
    _binding = None
    _load_error = exc


def __getattr__(name):
    if name == "binding" and _binding is not None:
        return _binding
    if name in _API:
        if _binding is None:
            raise ImportError(f"paper_2509_02753_amd: the HIP library is not usable ({_load_error}); build it with "
                              "`python -m paper_2509_02753_amd.build` -- there is no fallback implementation")
        return getattr(_binding, name)
    raise AttributeError(f"module 'paper_2509_02753_amd' has no attribute {name!r}")
