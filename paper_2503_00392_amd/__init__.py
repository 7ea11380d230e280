"""MI355X-native Progressive Sparse Attention decode path (arxiv 2503.00392).

The product is the C-ABI library ``libpsa.so`` (hand-written HIP for gfx950, declared in
``include/psa.h``).  This package is the thin Python binding over it: argument marshalling only.
"""
from .binding import (PSA_BF16, PSA_F16, SCORE_CUBOID_CENTER, SCORE_MEAN_KEY, SCORE_UPPER_BOUND, DecodeOutput, KvCache,
                      PsaError, Tier, Tuning, append_kv, build_block_means, build_block_metadata, decode_attention, decode_attention_static, decode_workspace_bytes, dense_attention, dense_workspace_bytes,
                      library_path, load_library, read_device_error, status_string, tier_init, tier_staging_bytes, tier_state_bytes,
                      tier_update, tier_update_workspace_bytes, topk_attention)

__all__ = ["PSA_BF16", "PSA_F16", "SCORE_CUBOID_CENTER", "SCORE_MEAN_KEY", "SCORE_UPPER_BOUND", "DecodeOutput", "KvCache",
           "PsaError", "Tier", "Tuning", "append_kv", "build_block_means", "build_block_metadata", "decode_attention", "decode_attention_static", "decode_workspace_bytes", "dense_attention", "dense_workspace_bytes",
           "library_path", "load_library", "read_device_error", "status_string", "tier_init", "tier_staging_bytes", "tier_state_bytes",
           "tier_update", "tier_update_workspace_bytes", "topk_attention"]
