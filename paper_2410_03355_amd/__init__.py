"""MI355X-native relaxed speculative-decoding verification (LANTERN, arXiv 2410.03355).

Python names mirror the C ABI of include/lantern.h: build_knn, verify,
verify_ex.  The work is done by hand-written gfx950 kernels in liblantern.so.
"""
from .binding import (  # noqa: F401
    BF16, F32, MAX_VOCAB, METRIC_COSINE, METRIC_L2, EXPORTS, LanternError, accept_chains, build_knn, build_knn_static,
    accept_trees, build_random, decide_rows, resample_selected, verify_trees, verify_trees_greedy, verify_trees_sequential,
    trees_sequential_workspace_bytes, knn_workspace_bytes, load, prepare, status_string, verify, verify_ex, verify_greedy,
    verify_greedy_rows, verify_rows,
)
from .build import LIB_PATH, build  # noqa: F401
