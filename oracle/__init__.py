"""CPU float64 oracle for chunk-based pre-filling attention and bi-level KV decoding.

THIS PACKAGE IS TEST INFRASTRUCTURE.  It is a plain, slow, definitional implementation used
only by tests, the smoke check and the CPU-baseline leg of the benchmark to judge the HIP
library.  It shares no code with the HIP path, imports nothing from it, and the product path
never calls it.

What it implements (paper: Method, "Efficiency Optimization"):
  * prefill  -- "Chunk-based Pre-filling" and the caption of its figure: every token of the
                chunk being processed attends to its own chunk (causally, the backbone being a
                decoder-only LLM), to the system prompt, and to the small kept set of tokens of
                every preceding chunk (the historical timestamp tokens).
  * score_topk, gather, decode -- "Bi-level KVs Decoding" and the caption of its figure: a
                relevance score per video chunk for the query, dense KVs reloaded for the most
                relevant chunks and sparse KVs for the others, all concatenated into one mixed
                KV set that generation attends to.

Every function is the mathematical definition written out with explicit score matrices in
float64; there is no tiling, no online softmax, no split/merge.  The paper prints no equations
and no worked numeric example for these steps, so the pins in tests/test_oracle_*.py are
invariants, closed forms, library special cases (torch CPU scaled_dot_product_attention) and
brute force on tiny inputs -- no function is pinned to a value printed in the paper.
"""
from .sets import allowed_mask, allowed_keys, allowed_pair_count, mixed_source_index
from .prefill import prefill_def, prefill_blk
from .bilevel import (chunk_scores, chunk_scores_mass, select_topk, gather_bilevel, decode_mixed, decode_lse,
                      pool_groups, pool_sparse_kv, gather_bilevel_pooled)

__all__ = [
    "allowed_mask", "allowed_keys", "allowed_pair_count", "mixed_source_index",
    "prefill_def", "prefill_blk",
    "chunk_scores", "chunk_scores_mass", "select_topk", "gather_bilevel", "decode_mixed", "decode_lse",
    "pool_groups", "pool_sparse_kv", "gather_bilevel_pooled",
]
