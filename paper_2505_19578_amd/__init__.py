"""SharePrefill prefill attention for AMD MI355X (gfx950).

The work is done by hand-written HIP kernels behind the C ABI declared in
``include/shareprefill.h`` (``libshareprefill.so``); this package is the thin
Python binding with the same entry-point names.  PyTorch is used only for
device memory and streams.  There is no CPU fallback: without the compiled
library (or without a GPU for the compute calls) the calls raise.
"""
from .binding import (SpError, SpShape, lib, shape_of, sp_workspace_bytes, sp_profile_enable, sp_profile_read,
                      sp_dense_attn_with_block_scores, sp_build_block_mask,
                      sp_block_sparse_attn, sp_prefill_layer, EXPORTED_SYMBOLS,
                      sp_score_workspace_bytes, sp_mask_workspace_bytes, sp_block_mean_logit_scores,
                      sp_build_block_mask_global, sp_build_block_mask_global_static, sp_prefill_layer_modes,
                      SP_STATIC_SCRATCH_BYTES,
                      sp_determine_pattern, sp_block_sparse_attn_gated, sp_prefill_layer_gated,
                      sp_prefill_layer_dict, pattern_dict_of, SpPatternDict,
                      sp_vs_workspace_bytes, sp_search_vertical_slash, SP_FALLBACK_DENSE, SP_FALLBACK_VERTICAL_SLASH,
                      SP_FALLBACK_VERTICAL_SLASH_TOKEN, sp_vs_token_workspace_bytes, sp_vertical_slash_attn,
                      SP_SCORE_BLOCK_MASS, SP_SCORE_MEAN_LOGIT, SP_SELECT_PER_ROW, SP_SELECT_GLOBAL,
                      )

__all__ = ["SpError", "SpShape", "lib", "shape_of", "sp_workspace_bytes", "sp_profile_enable", "sp_profile_read",
           "sp_dense_attn_with_block_scores", "sp_build_block_mask",
           "sp_block_sparse_attn", "sp_prefill_layer", "EXPORTED_SYMBOLS",
           "sp_score_workspace_bytes", "sp_mask_workspace_bytes", "sp_block_mean_logit_scores",
           "sp_build_block_mask_global", "sp_build_block_mask_global_static", "SP_STATIC_SCRATCH_BYTES",
           "sp_prefill_layer_modes",
           "sp_determine_pattern", "sp_block_sparse_attn_gated", "sp_prefill_layer_gated",
           "sp_prefill_layer_dict", "pattern_dict_of", "SpPatternDict",
           "sp_vs_workspace_bytes", "sp_search_vertical_slash", "SP_FALLBACK_DENSE", "SP_FALLBACK_VERTICAL_SLASH",
           "SP_FALLBACK_VERTICAL_SLASH_TOKEN", "sp_vs_token_workspace_bytes", "sp_vertical_slash_attn",
           "SP_SCORE_BLOCK_MASS", "SP_SCORE_MEAN_LOGIT", "SP_SELECT_PER_ROW", "SP_SELECT_GLOBAL",
           ]
