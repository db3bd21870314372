"""Exact brute-force k-nearest-neighbour search for AMD MI355X (gfx950).

`knn_build` / `knn_search` are thin bindings over the C ABI of libknn.so
(include/knn.h); the work is done by hand-written HIP kernels.  Build the
library with `python -m paper_0906_0231_amd.build`.
"""
from .api import (KNN_COSINE, KNN_MAX_K, KNN_SQEUCLIDEAN, KnnError, KnnResult, knn_build,
                  knn_mfma_calibration, knn_mfma_bf16_calibration, knn_contraction_calibration, knn_read_calibration, knn_search, knn_search_static, knn_valu_calibration, knn_select, knn_workspace_bytes, knn_workspace_bytes_min, knn_plan, load_library)

__all__ = ["knn_build", "knn_search", "knn_search_static", "knn_select", "knn_mfma_calibration", "knn_mfma_bf16_calibration", "knn_contraction_calibration", "knn_valu_calibration", "knn_read_calibration", "knn_workspace_bytes", "knn_workspace_bytes_min", "knn_plan", "load_library", "KnnError",
           "KnnResult", "KNN_SQEUCLIDEAN", "KNN_COSINE", "KNN_MAX_K"]
