"""PoD attention over a split KV cache for MI355X (gfx950): thin Python binding of libpod.so."""
from .binding import (  # noqa: F401
    EXPORTS, PodCache, PodConfig, PodError, load, lib_path, make_config, pod_cache_bytes,
    pod_cache_live_bytes, pod_group_layers, pod_layer_similarity, pod_prefill_chunk_workspace_bytes, pod_prefill_chunk_in_place_bytes, pod_score_buffer_bytes,
    pod_workspace_bytes, pod_profile_stream_read, guarded_empty, guards_intact, pod_profile_mfma_feed, pod_decode_plan, pod_decode_even_plan,
    pod_select_workspace_bytes, POOL_AVG, POOL_MAX,
)
