"""MI355X-native batched graph retrieval with a learned MLP relevance (arXiv 2502.11490).

Thin ctypes binding over the C ABI in include/gmpgr_ann.h.  Functions have the names of the
C entry points and only marshal arguments: every step of the search runs in the HIP kernels
of libgmpgr_ann.so.  There is no CPU fallback; importing works without a GPU, calling does not.
"""
from .binding import (  # noqa: F401
    ANN_BF16,
    ANN_F8,
    ANN_F16,
    ANN_F32,
    ANN_MLP_GENERIC,
    ANN_VALIDATE,
    AnnError,
    Graph,
    Mlp,
    Stats,
    ann_graph_load,
    ann_last_error,
    ann_mlp_load,
    ann_mlp_uses_mfma,
    ann_profile_copy,
    ann_profile_enable,
    ann_profile_read,
    ann_score_pairs,
    ann_score_pairs_noalloc,
    ann_users_add_noise,
    ann_quantize_e4m3,
    ann_search,
    ann_search_layers,
    ann_search_layers_workspace_bytes,
    ann_search_ragged,
    ann_search_stream,
    ann_stream_open,
    Stream,
    ann_search_walkers,
    ann_search_walkers_workspace_bytes,
    ann_search_stream_workspace_bytes,
    ann_search_stats,
    ann_set_progress_timeout,
    ann_search_workspace_bytes,
    lib_path,
    load_library,
)
