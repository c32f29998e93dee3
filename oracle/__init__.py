"""CPU oracle for the expert-pruning hot path (TEST INFRASTRUCTURE ONLY).

Plain, slow, fp64 numpy implementations of what the GPU library computes,
written from the paper's definitions (Sec. 3.1 Eq. 1-2, Sec. 3.2 Eq. 3,
Sec. 3.3, App. A.2).  Nothing here is tuned and nothing here is part of the
product: only the tests, the smoke check and the benchmark's `cpu_baseline`
leg may import this package.  It shares no code with the HIP path and does
not import the GPU package.
"""
from .moe_reference import (  # noqa: F401
    silu,
    expert_ffn,
    expert_outputs,
    routing_order,
    renormalised_weights,
    layer_output,
    kept_subsets,
    subset_mask,
    pruned_layer_output,
    prune_enumerate,
    prune_enumerate_streamed,
    prune_enumerate_gram_form,
    skip_decision,
    forward_skip,
    median_skip_ratio,
    skip_topk_decision,
    forward_skip_topk,
    expert_selection_stats,
    frequency_kept,
)
from .brute_force import brute_force_enumerate  # noqa: F401
