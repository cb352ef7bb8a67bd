"""MI355X-native two-stage diversified graph (TSDG) build and best-first k-NN
search.  All computation happens in the HIP library (csrc/, C ABI declared in
include/tsdg_ann.h); this package only marshals arguments.  There is no CPU
fallback: calls raise if the library cannot be loaded."""
from .api import (  # noqa: F401
    ANN_F32, ANN_U8, ANN_F16, ANN_L2, ANN_COSINE, AnnError, ann_normalize_rows, ann_max_row_norm, ann_ip_augment_rows, Graph, QueryStats, ann_bruteforce, ann_build_graph, ann_build_graph_ex,
    ann_graph_export, ann_graph_free, ann_graph_import, ann_graph_info, ann_knn, ann_knn_descent, ann_last_error, ann_probe_gather, ann_probe_mfma,
    ann_search, ann_search_ex, ann_search_multi, ann_search_multi_static, ann_search_multi_workspace_bytes, ann_search_alg2, library_path, load_library,
)
