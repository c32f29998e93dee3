"""MI355X-native expert-subset scoring and dynamic skipping for one MoE layer.

The compute path is the C-ABI library `libmoeprune.so` (hand-written HIP for
gfx950); `binding` marshals torch tensors into it and nothing else.  Importing
`binding` (or any name re-exported from it) fails loudly when the library has
not been built -- there is no CPU fallback.  `workloads` only draws seeded
synthetic inputs and can be imported on its own.
"""
_BINDING_NAMES = (
    "moe_expert_outputs", "prune_enumerate", "prune_enumerate_multi", "prune_enumerate_static", "prune_enumerate_direct",
    "moe_forward_skip", "moe_forward_pruned_skip",
    "moe_pack_weights", "moe_forward_pruned_skip_packed", "moe_expert_outputs_packed",
    "moe_forward_skip_topk", "skip_calibrate_beta", "expert_selection_stats",
    "moe_expert_outputs_ranked", "prune_enumerate_ranked",
    "num_subsets", "subset_unrank", "subset_rank", "library_path", "MoepError",
    "kernel_timing_enable", "kernel_timing_collect", "kernel_timing_reset", "kernel_timing_records", "mfma_ceiling",
)


def __getattr__(name):
    if name in _BINDING_NAMES or name == "binding":
        import importlib

        mod = importlib.import_module(".binding", __name__)
        return mod if name == "binding" else getattr(mod, name)
    raise AttributeError(f"module {__name__!r} has no attribute {name!r}")
