"""MI355X-native BigBird block-sparse attention (Sec. 2 eq. (AT), App. D).

Thin Python binding over the C ABI of include/bigbird.h.  All computation runs in
the HIP kernels of libbigbird.so; PyTorch only supplies device memory and streams.
There is no CPU fallback: a missing library raises.
"""
from .binding import (BB_BF16, BB_F32, BB_GLOBAL_FIRST_LAST, BB_GLOBAL_LEADING,
                      BB_SKIP_PADDED_QUERY_BLOCKS, BigBirdError,
                      EXPORTED_SYMBOLS, bigbird_attn_bwd, bigbird_attn_bwd_dropout, bigbird_attn_fwd,
                      bigbird_attn_fwd_dropout, bigbird_attn_fwd_static, bigbird_dropout_keep_mask,
                      bigbird_attn_workspace_bytes, bigbird_count_block_pairs,
                      bigbird_make_rand_idx, bigbird_status_string, bigbird_validate_rand_idx,
                      library_path, load_library, prepare_attn_bwd, prepare_attn_fwd)

__all__ = [
    "BB_BF16", "BB_F32", "BB_GLOBAL_FIRST_LAST", "BB_GLOBAL_LEADING", "BB_SKIP_PADDED_QUERY_BLOCKS",
    "BigBirdError",
    "EXPORTED_SYMBOLS", "bigbird_attn_bwd", "bigbird_attn_bwd_dropout", "bigbird_attn_fwd",
    "bigbird_attn_fwd_dropout", "bigbird_attn_fwd_static", "bigbird_dropout_keep_mask",
    "bigbird_attn_workspace_bytes",
    "bigbird_count_block_pairs", "bigbird_make_rand_idx", "bigbird_status_string",
    "bigbird_validate_rand_idx", "library_path", "load_library", "prepare_attn_bwd", "prepare_attn_fwd",
]
