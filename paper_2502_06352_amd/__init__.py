"""MI355X-native static-tree relaxed verification (LANTERN++ hot path).

The product is ``liblpp.so`` (hand-written HIP for gfx950, C ABI in
``include/lpp.h``); this package is its thin ctypes binding.
"""
from .binding import (  # noqa: F401
    LIB_PATH, LPP_BF16, LPP_F32, LPP_OK, LPP_EINVAL, LPP_EUNSUPPORTED, LPP_ENOWORKSPACE, LPP_EHIP,
    LppError, Tree, lib,
    lpp_build_neighbours, lpp_build_neighbours_workspace,
    lpp_tree_attention, lpp_tree_attention_gqa, lpp_tree_attention_workspace,
    lpp_tree_attention_layers, lpp_tree_attention_layers_workspace,
    lpp_relaxed_verify, lpp_relaxed_verify_workspace, lpp_relaxed_verify_additive, lpp_relaxed_verify_static,
    lpp_commit_kv, lpp_probe_stream_read, lpp_relaxed_verify_sampled, lpp_relaxed_verify_opts,
    LPP_BOUND_MULTIPLICATIVE, LPP_BOUND_ADDITIVE, LPP_RULE_PREFIX, LPP_RULE_SKIP,
    LPP_SIBLINGS_IID, LPP_SIBLINGS_DISTINCT,
)
