"""MI355X-native hot path of one Medusa verification step (arXiv 2401.10774).

The work is done by hand-written gfx950 HIP kernels behind the C ABI of include/medusa.h
(libmedusa_hip.so, built in-tree by `paper_2401_10774_amd.build`).  This package is the thin
binding with the same entry-point names.
"""
from .binding import (
    MedusaError,
    MedusaTree,
    kv_commit,
    lib,
    library_path,
    medusa_accept,
    medusa_accept_sampled,
    medusa_accept_fused,
    medusa_verify_fused_available,
    medusa_verify_logits,
    medusa_accept_workspace_bytes,
    medusa_carry_over,
    medusa_heads,
    medusa_gemm_plan,
    medusa_topk_tree,
    tree_attention,
    tree_attention_static,
    tree_attention_workspace_bytes,
    interleave_gate_up,
    tree_linear,
    tree_linear_segments,
    tree_linear_swiglu,
    tree_linear_workspace_bytes,
    tree_rope,
)

__all__ = [
    "MedusaError", "MedusaTree", "kv_commit", "lib", "library_path", "medusa_accept", "medusa_accept_sampled", "medusa_accept_fused", "medusa_verify_fused_available", "medusa_verify_logits",
    "medusa_accept_workspace_bytes", "medusa_carry_over", "medusa_heads", "medusa_gemm_plan", "medusa_topk_tree", "tree_attention",
    "tree_attention_workspace_bytes", "tree_attention_static", "tree_linear", "tree_linear_segments", "tree_linear_swiglu", "interleave_gate_up",
    "tree_linear_workspace_bytes", "tree_rope",
]
