"""MI355X (gfx950) implementation of the PLAID search path behind the C ABI of include/plaid.h.

`plaid.py` is the ctypes binding (same names as the header); `build.py` compiles csrc/*.hip into
libplaid.so in-tree.  Nothing here imports the CPU oracle.
"""
from .plaid import (  # noqa: F401
    EXPORTS,
    Index,
    PlaidError,
    load_library,
    plaid_assign_centroids,
    plaid_build_ivf,
    plaid_decompress_passages,
    plaid_encode_residuals,
    plaid_get_score_kernel,
    plaid_get_score_kernel_clocks,
    plaid_index_set_renormalize,
    plaid_get_stage2_kernel,
    plaid_get_stage_ms,
    plaid_index_free,
    plaid_index_from_view,
    plaid_index_info,
    plaid_index_load,
    plaid_last_error,
    plaid_search,
    plaid_search_debug,
    plaid_search_static,
    plaid_search_vanilla,
    plaid_set_max_chunk,
    plaid_set_stage_timing,
    plaid_workspace_bytes,
)
