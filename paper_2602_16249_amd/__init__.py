"""MI355X-native neighbourhood attention for AFFMAE's off-grid backbone.

The compute lives in libaffmae.so (hand-written HIP for gfx950, C ABI declared
in include/affmae.h).  This package is the thin Python binding: it marshals
torch device tensors into that ABI and owns no arithmetic.  There is no CPU or
PyTorch fallback: without the built library every call raises.
"""
from .binding import (  # noqa: F401
    AffmaeError,
    affmae_cluster,
    affmae_knn,
    affmae_knn_static,
    affmae_merge_bwd,
    affmae_merge_fwd,
    affmae_merge_select,
    affmae_pla_bwd,
    affmae_pla_bwd_relpos,
    affmae_pla_fwd,
    affmae_pla_fwd_relpos,
    affmae_pla_plan,
    affmae_vts_bwd,
    affmae_vts_fwd,
    affmae_vts_table,
    build_id,
    library_path,
    load_library,
    status_string,
    timing_enable,
    timing_read,
    timing_reset,
    use_timed_library,
)

__all__ = ["AffmaeError", "affmae_cluster", "affmae_knn", "affmae_knn_static", "affmae_merge_select", "affmae_merge_fwd", "affmae_merge_bwd", "affmae_pla_fwd", "affmae_pla_bwd", "affmae_pla_plan", "affmae_pla_fwd_relpos", "affmae_pla_bwd_relpos", "affmae_vts_table", "affmae_vts_fwd", "affmae_vts_bwd", "library_path", "load_library",
           "status_string"]
