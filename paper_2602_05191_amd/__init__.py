"""MI355X-native Double-P decode attention (hierarchical top-p sparse attention
over a clustered KV cache): hand-written gfx950 kernels behind a C ABI
(include/dp.h) and a thin ctypes binding with the same entry-point names."""
from .binding import (  # noqa: F401
    DP_BF16,
    DP_CLUSTER_PINNED,
    DP_F32,
    DP_FLAG_P2_ABSOLUTE,
    DPError,
    DeviceCache,
    Prefill,
    Problem,
    dp_budget_decode_attention,
    dp_build_cluster_cache,
    dp_build_workspace_bytes,
    dp_decode_attention,
    dp_decode_attention_timed,
    dp_dense_decode,
    dp_score_centroids,
    dp_score_centroids_timed,
    dp_sparse_decode,
    dp_topk_select,
    dp_topp_select,
    dp_topp_select_sorted,
    dp_workspace_bytes,
    dp_workspace_layout,
    library_path,
    load_library,
)
