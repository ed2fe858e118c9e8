"""CPU oracle (test infrastructure): see specattn_oracle.c for what it computes.

Only tests/, the smoke check and the bench's cpu_baseline leg may import this
package.  It never imports the HIP binding.
"""
from .layer_map import layer_map, layer_map_exhaustive, layer_similarity, layer_similarity_fast, monotone_maps  # noqa: F401
from .oracle import (  # noqa: F401
    ROW_INVALID,
    ROW_NEAR_BOUNDARY,
    SelectResult,
    UnionResult,
    bisection_select,
    chunk_masses,
    chunk_token_mask,
    masked_attention,
    nucleus_bisection,
    set_threads,
    topp_select,
    topp_select_chunks,
    topp_select_union,
)
