"""MI355X-native lightning-indexer top-k (StreamIndex hot path).

The product is libstreamindex.so (HIP, gfx950) behind the C ABI of include/streamindex.h;
this package is its thin Python binding.  Importing the package does not load the library;
the first call does, and fails loudly if it has not been built."""
from .binding import (  # noqa: F401
    EXPORTS, LIB_PATH, PHASE_NAMES, PHASE_TIME_WORDS, PHASE_TRACE_EVENTS, PHASE_WORDS, PROFILE_CLASS_NAMES, SI_ERR_HIP, SI_ERR_INVALID_ARG,
    SI_ERR_UNSUPPORTED_SHAPE, SI_ERR_WORKSPACE_TOO_SMALL, SI_MASK_CAUSAL_BLOCK, SI_MASK_NONE,
    SI_OK, StreamIndexError, load, si_fused_workspace_bytes, si_indexer_topk, si_fused_shape_for, si_indexer_topk_fused, si_indexer_topk_fused_shape, si_indexer_topk_static,
    si_indexer_topk_tiled, si_last_hip_error,
    si_materialize_bytes, si_plan_tiles, si_profile_enable, si_profile_phases, si_profile_read, si_profile_reset,
    si_score_tile, si_sparse_attention, si_strerror, si_topk_from_scores, si_version, si_wall_clock_khz, si_workspace_bytes,
)
