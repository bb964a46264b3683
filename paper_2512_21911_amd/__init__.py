"""libsvf: sparse verification attention for speculative decoding, native to AMD MI355X (gfx950).

The product is the C-ABI library built from csrc/ (declared in include/svf.h); this package is
its thin ctypes binding.
"""
from .binding import (SVF_BF16, SVF_F32, SVF_STEP_ANCHOR, SVF_STEP_REUSE, SVF_STEP_REUSE_GATHER, SvfError, SvfShape, lib, make_shape, new_workspace, strerror,  # noqa: F401
                      svf_block_reps, svf_budget_blocks, svf_score_select, svf_workspace_set_wait_polls, svf_static_workspace_bytes, svf_verify_attn_static_ws, SVF_KERNEL_AUTO, SVF_KERNEL_VECTOR_ALU, new_diag_workspace, svf_diag_verify_attn, svf_diag_wait_fallbacks, svf_verify_attn, svf_verify_step,
                      svf_version, svf_workspace_bytes, svf_workspace_init,
                      new_analytics_workspace, svf_jaccard_adjacent, svf_mask_words, svf_masks_from_selection,
                      svf_overlap_by_distance, svf_select_per_draft, svf_topk_anchors,
                      SVF_BUDGET_GLOBAL, SVF_BUDGET_PER_HEAD, SVF_GROUP_MAX, SVF_GROUP_MEAN, SVF_SUMMARY_MEAN,
                      SVF_SUMMARY_MINMAX, SvfRetrieval, svf_block_summaries, svf_retrieve,
                      SVF_ACT_GELU, SVF_ACT_SILU, SVF_FFN_WALK_AUTO, SVF_FFN_WALK_GATE_FIRST, SVF_FFN_WALK_TOGETHER, SvfFfnShape, make_ffn_shape, new_ffn_workspace,
                      svf_ffn_workspace_bytes, svf_sparse_ffn,
                      svf_accept_resample, svf_moe_calibrate, svf_moe_skip)
