"""MI355X-native ClusterKV hot path: thin Python binding over libclusterkv.so.

Every step of the path (K-means assignment/update, metadata, cluster selection,
index gather, sparse decode attention) runs in the HIP kernels of the C-ABI
library declared in include/clusterkv.h.  This package only marshals torch
tensors (device memory, current stream) into those calls.  There is no CPU or
PyTorch fallback: a missing library is an error.
"""
from .binding import (CK_BF16, CK_F32, CK_KM_UNTIL_CONVERGED, CK_METRIC_COSINE, CK_METRIC_IP,
                      CK_METRIC_L2, CK_SEL_TRIM_LAST, CK_SEL_WHOLE, CK_MAX_CLUSTERS,
                      ClusterCache, ClusterKVError, ClusterState, Shape, cached_decode_step,
                      ck_cache_reset, ck_cached_decode_step, ck_host_device_ptr, ck_build_metadata, ck_cluster_keys,
                      ck_cluster_keys_opt,
                      ck_decode_step, ck_expand_pages, ck_full_decode_attn, ck_gather_indices,
                      ck_kmeans_assign, ck_kmeans_objective, ck_kmeans_update, ck_page_keys, ck_probe_mfma_bf16,
                      ck_recall_hits, ck_select_clusters, ck_sparse_decode_attn,
                      ck_sparse_decode_attn_static, ck_token_scores,
                      ck_topk_select, ck_version, ck_workspace_bytes, decode_step, load_library)
from .driver import LayerStack

__all__ = [
    "LayerStack",
    "CK_BF16", "CK_F32", "CK_KM_UNTIL_CONVERGED", "CK_METRIC_COSINE", "CK_METRIC_IP",
    "CK_METRIC_L2", "CK_SEL_TRIM_LAST", "CK_SEL_WHOLE", "CK_MAX_CLUSTERS", "ck_cluster_keys_opt",
    "ClusterCache", "ClusterKVError", "ClusterState", "Shape", "cached_decode_step",
    "ck_cache_reset", "ck_cached_decode_step", "ck_host_device_ptr", "ck_build_metadata", "ck_cluster_keys",
    "ck_decode_step", "ck_expand_pages", "ck_full_decode_attn", "ck_gather_indices",
    "ck_kmeans_assign", "ck_kmeans_objective", "ck_kmeans_update", "ck_page_keys", "ck_probe_mfma_bf16",
    "ck_recall_hits", "ck_select_clusters", "ck_sparse_decode_attn",
    "ck_sparse_decode_attn_static", "ck_token_scores",
    "ck_topk_select", "ck_version", "ck_workspace_bytes", "decode_step", "load_library",
]
