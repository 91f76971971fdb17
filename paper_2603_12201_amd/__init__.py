"""MI355X-native IndexCache / DeepSeek-Sparse-Attention hot path.

Thin Python binding (argument marshalling only) over libindexcache.so, the hand-written
HIP library declared in include/indexcache.h.  Every step of the path runs in that library;
there is no CPU or PyTorch fallback: if the library is missing, loading fails loudly.
PyTorch is used for device memory and streams only.
"""
from .binding import (  # noqa: F401
    IcError, Status, lib, lib_path, last_error,
    indexer_topk, indexer_topk_workspace, sparse_attn, sparse_attn_workspace, sparse_attn_static, STATIC_SCRATCH_BYTES,
    forward_stack, forward_stack_workspace, make_layers,
    pattern_from_string, pattern_uniform, topk_overlap,
    cosine_rows, similarity_matrix, pattern_search_dp,
    pattern_search_greedy, pattern_loss, greedy_search_forward,
    attn_probs, distill_loss,
    paged_cache, indexer_topk_paged, sparse_attn_paged, forward_stack_paged,
    debug_indexer_scores, debug_indexer_launch_count,
    prof_enable, prof_collect, prof_get, prof_reset,
    calibrate, CALIB_READ, CALIB_COPY, CALIB_GATHER, CALIB_MFMA_BF16, CALIB_MFMA_FP8,
    CALIB_TILE_GATHER, CALIB_TILE_STORE, CALIB_TILE_READ, CALIB_TILE_READ2, CALIB_TILE_8WAVES, CALIB_TILE_INTERLEAVED,
    CALIB_LDS_READ16_PADDED, CALIB_LDS_READ16_SWIZZLED, CALIB_LDS_TR8_ROWS2, CALIB_LDS_TR8_ROWS1,
    IndexerDesc, AttnDesc, Layer, PagedCache,
)
