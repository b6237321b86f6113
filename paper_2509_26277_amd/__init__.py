"""MI355X-native hot path of CAT (Cluster-based Affine Transformation).

``cat_fit`` / ``cat_apply`` and the step-level calls are thin ctypes wrappers over
the C-ABI library ``libcat_hip.so`` (hand-written HIP for gfx950).  Importing this
package does not load the library; the first call does, and it fails loudly if
the library has not been built.  ``workloads`` holds the seeded input generators.
"""
from .binding import (  # noqa: F401
    CatError,
    cat_fit,
    cat_apply,
    cat_apply_static,
    cat_assign,
    cat_update,
    cat_stats,
    cat_init_indices,
    cat_pca_fit,
    cat_pca_project,
    cat_apply_assigned,
    cat_fit_pca,
    cat_apply_pca,
    cat_alpha_sweep,
    cat_top1,
    cat_init_kmeanspp,
    cat_fit_restarts,
    cat_fit_multi_k,
    cat_params_to_bf16,
    cat_apply_lp,
    cat_fit_workspace_bytes,
    cat_apply_workspace_bytes,
    library_path,
    load_library,
)
