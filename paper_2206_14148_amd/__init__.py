"""MI355X-native exact brute-force kNN and kernel matrix-vector product under a caller-given
device-memory limit.

The package is a thin binding over libknn_mi355x.so (include/knn.h, include/kmv.h); see
binding.py.
"""
from .binding import (  # noqa: F401
    KNN_ERR_HIP, KNN_ERR_INVALID_ARG, KNN_ERR_MEM_LIMIT_TOO_SMALL, KNN_ERR_UNSUPPORTED,
    KNN_ERR_WORKSPACE_TOO_SMALL, KNN_MAX_K, KNN_METRIC_COSINE, KNN_METRIC_L1, KNN_METRIC_L2SQ, KNN_OK, KNN_PATH_L1, KNN_PATH_LOWD, KNN_PATH_LOWD_MFMA, KNN_PATH_LOWD_BF16, KNN_PATH_MFMA_SPLIT, KNN_PATH_MFMA_PACKED, KNN_PATH_MFMA_WIDE,
    EXPORTED_SYMBOLS, KnnError, Plan, knn_chunk_rows, knn_last_stats, knn_parse_size, knn_plan, knn_profile_enable,
    knn_profile_read,
    KMV_PATH_LOWD, KMV_PATH_MFMA, KMV_PATH_VALU, KmvPlan, kmv_apply, kmv_apply_raw, kmv_plan,
    HostPlan, knn_plan_host_x, knn_search_host_x, SgprPlan, sgpr_accumulate, sgpr_plan,
    KNN_ERR_STATIC_SCRATCH_TOO_SMALL, KNN_STATIC_SCRATCH_BYTES, knn_search_static, knn_measure_mfma_peak,
    knn_search, knn_search_raw, knn_status_string, knn_workspace_bytes, library_path, load,
)
