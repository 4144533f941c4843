"""CPU oracle for BigBird block-sparse attention.  TEST INFRASTRUCTURE ONLY.

Plain, slow, fp64 NumPy code that evaluates the paper's definition directly: it
builds the dense n x n adjacency matrix A of the BigBird graph (Sec. 2 and
App. D) and computes masked softmax attention, eq. (AT) per head, from it.  It
shares no code with the HIP library and must never be imported by the product
package: only the tests, the smoke check and the benchmark's CPU-baseline leg
may call it.

Pin status (see tests/test_oracle_pins.py): every function here is pinned by
something other than itself -- full coverage equals textbook attention computed
by an independent per-element loop, closed forms for Q = 0, row/column counts of
the pattern ((g+w+r) b keys per interior row, App. D), brute force over an
explicit edge list at the paper's figure sizes, central finite differences for
the gradients.  What is NOT pinned is agreement with the authors' released
code on points the paper leaves open (how random blocks are drawn, whether
overlapping components are counted once): "parity unpinned" for those readings.
The ETC construction (etc.py: extra global tokens in front of the sequence) is pinned in
tests/test_oracle_etc_pins.py: against the ITC functions where the two constructions coincide,
by an independent per-element loop, by row counts at the paper's ETC sizes, by closed forms and
by finite differences.
Attention dropout (dropout.py: the keep mask is a counter-based function of seed, slice, query and
key) is pinned in tests/test_oracle_dropout_pins.py; agreement with the authors' own dropout
stream is "parity unpinned" (the paper fixes only the rate).
"""
from .pattern import (GLOBAL_FIRST_LAST, GLOBAL_LEADING, global_blocks, window_blocks,
                      make_rand_idx, validate_rand_idx, neighbour_blocks, dense_block_mask,
                      dense_mask, count_block_pairs, reverse_random_lists)
from .attention import attn_fwd, attn_bwd, attn_fwd_rows
from .etc import dense_mask_etc, attn_fwd_etc, attn_bwd_etc
from .dropout import attn_fwd_dropout, attn_fwd_dropout_rows, attn_bwd_dropout, keep_mask, dropout_threshold, dropout_scale

__all__ = [
    "GLOBAL_FIRST_LAST", "GLOBAL_LEADING", "global_blocks", "window_blocks", "make_rand_idx",
    "validate_rand_idx", "neighbour_blocks", "dense_block_mask", "dense_mask",
    "count_block_pairs", "reverse_random_lists", "attn_fwd", "attn_bwd", "attn_fwd_rows",
    "dense_mask_etc", "attn_fwd_etc", "attn_bwd_etc",
    "attn_fwd_dropout", "attn_fwd_dropout_rows", "attn_bwd_dropout", "keep_mask", "dropout_threshold", "dropout_scale",
]
