"""CPU oracle for the CAT hot path (test infrastructure, never the product path).

Thin ctypes access to ``cat_oracle.c`` (plain C, IEEE double).  Nothing in this
package imports, links or calls the GPU library; the GPU library never imports
this package.  Allowed callers: ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py``.
"""
from .cat_oracle import (  # noqa: F401
    build,
    threads,
    splitmix64,
    init_indices,
    assign,
    distances,
    update,
    affine,
    fit,
    apply,
    covariance,
    pca_fit,
    pca_project,
    alpha_sweep,
    kmeanspp,
    fit_restarts,
    fit_early_stop,
    fit_multi_k,
    to_bf16,
    apply_lp,
    fit_bounds,
)
