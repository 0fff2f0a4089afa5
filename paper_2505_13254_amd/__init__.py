"""MI355X-native tree-verification hot path of heterogeneity-adaptive speculative decoding.

The product is libheterospec.so (hand-written HIP for gfx950 behind a C ABI, see
include/heterospec.h); this package is its thin Python binding.
"""
_BINDING = ("hs_draft_entropy_topk", "hs_workspace_prepare", "hs_tree_prune", "hs_tree_prune_static", "hs_tree_attention", "hs_verify_accept", "hs_tree_expand",
            "hs_adaptive_control", "hs_adaptive_policy", "hs_kv_commit", "hs_kv_commit_paged", "hs_tree_attention_paged", "hs_tree_validate", "hs_time_next_attention", "hs_tree_attention_last_kernel", "hs_tree_attention_plan", "new_tree_state", "HS_PSTAR_CUMULATIVE", "HS_PSTAR_LOCAL", "lib",
            "HsError", "HS_F32", "HS_BF16", "HS_ACCEPT_GREEDY", "HS_ACCEPT_STOCHASTIC",
            "HS_ACCEPT_STOCHASTIC_POINTMASS", "HS_MAX_TOPK", "LIB_PATH", "exported_symbols", "workspace")


def __getattr__(name):
    if name in _BINDING:
        from . import binding
        return getattr(binding, name)
    raise AttributeError(name)
