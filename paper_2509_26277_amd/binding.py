"""ctypes binding of ``libcat_hip.so`` (the C ABI declared in ``include/cat.h``).

Argument marshalling only: every step of the path runs in the HIP kernels.
PyTorch is used for device memory and the stream handle.  There is no CPU
fallback: if the library is missing the first call raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libcat_hip.so")
_lib = None

CAT_F32, CAT_BF16 = 0, 1
CAT_PATH_AUTO, CAT_PATH_STREAM, CAT_PATH_TILE = 0, 1, 2
_STATUS = {0: "CAT_OK", 1: "CAT_ERR_INVALID_ARG", 2: "CAT_ERR_UNSUPPORTED", 3: "CAT_ERR_WORKSPACE",
           4: "CAT_ERR_DEVICE"}

EXPORTS = ("cat_select_path", "cat_fit_workspace_bytes", "cat_apply_workspace_bytes", "cat_fit", "cat_apply",
           "cat_assign", "cat_update", "cat_stats", "cat_init_indices", "cat_last_error", "cat_profile_enable",
           "cat_profile_read", "cat_debug_list_capacity", "cat_debug_rerank_queue", "cat_pca_workspace_bytes", "cat_pca_fit", "cat_pca_project",
           "cat_apply_assigned", "cat_fit_pca_workspace_bytes", "cat_fit_pca", "cat_apply_pca_workspace_bytes", "cat_apply_pca",
           "cat_alpha_sweep_workspace_bytes", "cat_alpha_sweep", "cat_top1",
           "cat_init_kmeanspp_workspace_bytes", "cat_init_kmeanspp",
           "cat_fit_restarts_workspace_bytes", "cat_fit_restarts", "cat_fit_early_stop", "cat_allow_early_stop",
           "cat_apply_static", "cat_apply_static_max_workspace_bytes", "cat_debug_apply_kernel",
           "cat_fit_multi_k_workspace_bytes", "cat_fit_multi_k", "cat_debug_multi_group_tiles",
           "cat_params_to_bf16", "cat_apply_lp_workspace_bytes", "cat_apply_lp",
           "cat_fit_bounds_workspace_bytes", "cat_fit_bounds", "cat_debug_padded_fit", "cat_stream_probe")


class CatError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"{_STATUS.get(status, status)}: {message}")
        self.status = status


def library_path():
    return _SO


def load_library():
    """Load libcat_hip.so (built by ``python -m paper_2509_26277_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_SO):
        raise RuntimeError(f"{_SO} is not built; run `python -m paper_2509_26277_amd.build` "
                           "(there is no fallback path)")
    lib = ctypes.CDLL(_SO)
    c = ctypes
    vp, i64, i32, u64, sz = c.c_void_p, c.c_int64, c.c_int32, c.c_uint64, c.c_size_t
    lib.cat_select_path.argtypes = [c.c_int]
    lib.cat_select_path.restype = c.c_int
    lib.cat_fit_workspace_bytes.argtypes = [i64, i64, i32, c.c_int]
    lib.cat_fit_workspace_bytes.restype = sz
    lib.cat_apply_workspace_bytes.argtypes = [i64, i64, i32, c.c_int]
    lib.cat_apply_workspace_bytes.restype = sz
    lib.cat_fit.argtypes = [vp, vp, i64, i64, i32, i32, u64, c.c_int, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.cat_fit.restype = c.c_int
    lib.cat_fit_early_stop.argtypes = [vp, vp, i64, i64, i32, i32, u64, c.c_int, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.cat_fit_early_stop.restype = c.c_int
    lib.cat_allow_early_stop.argtypes = [c.c_int]
    lib.cat_allow_early_stop.restype = c.c_int
    lib.cat_apply.argtypes = [vp, i64, i64, i32, c.c_int, vp, vp, vp, c.c_float, vp, vp, vp, sz, vp]
    lib.cat_apply.restype = c.c_int
    lib.cat_apply_static.argtypes = [vp, i64, i64, i32, c.c_int, vp, vp, vp, c.c_float, vp, vp, vp]
    lib.cat_apply_static.restype = c.c_int
    lib.cat_apply_static_max_workspace_bytes.argtypes = []
    lib.cat_apply_static_max_workspace_bytes.restype = sz
    lib.cat_assign.argtypes = [vp, i64, i64, i32, c.c_int, vp, vp, vp, vp, vp, sz, vp]
    lib.cat_assign.restype = c.c_int
    lib.cat_update.argtypes = [vp, vp, i64, i64, i32, c.c_int, vp, vp, vp, vp, sz, vp]
    lib.cat_update.restype = c.c_int
    lib.cat_stats.argtypes = [vp, vp, vp, i64, i64, i32, c.c_int, vp, vp, vp, vp, vp, sz, vp]
    lib.cat_stats.restype = c.c_int
    lib.cat_init_indices.argtypes = [i64, i32, u64, c.POINTER(c.c_int64)]
    lib.cat_init_indices.restype = c.c_int
    lib.cat_profile_enable.argtypes = [c.c_int]
    lib.cat_profile_enable.restype = c.c_int
    lib.cat_profile_read.argtypes = [c.POINTER(c.c_float), c.c_int]
    lib.cat_profile_read.restype = c.c_int
    lib.cat_pca_workspace_bytes.argtypes = [i64, i64, i32, c.c_int]
    lib.cat_pca_workspace_bytes.restype = sz
    lib.cat_pca_fit.argtypes = [vp, i64, i64, i32, c.c_int, i32, vp, vp, vp, vp, sz, vp]
    lib.cat_pca_fit.restype = c.c_int
    lib.cat_pca_project.argtypes = [vp, i64, i64, i32, c.c_int, vp, vp, vp, vp]
    lib.cat_pca_project.restype = c.c_int
    lib.cat_apply_assigned.argtypes = [vp, vp, i64, i64, i32, c.c_int, vp, vp, c.c_float, vp, vp]
    lib.cat_apply_assigned.restype = c.c_int
    lib.cat_fit_pca_workspace_bytes.argtypes = [i64, i64, i32, i32, c.c_int]
    lib.cat_fit_pca_workspace_bytes.restype = sz
    lib.cat_fit_pca.argtypes = [vp, vp, i64, i64, i32, i32, i32, u64, c.c_int, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.cat_fit_pca.restype = c.c_int
    lib.cat_apply_pca_workspace_bytes.argtypes = [i64, i64, i32, i32, c.c_int]
    lib.cat_apply_pca_workspace_bytes.restype = sz
    lib.cat_apply_pca.argtypes = [vp, i64, i64, i32, i32, c.c_int, vp, vp, vp, vp, vp, c.c_float, vp, vp, vp, sz, vp]
    lib.cat_apply_pca.restype = c.c_int
    lib.cat_alpha_sweep_workspace_bytes.argtypes = []
    lib.cat_alpha_sweep_workspace_bytes.restype = sz
    lib.cat_alpha_sweep.argtypes = [vp, vp, vp, vp, i64, i64, i32, c.c_int, vp, vp, c.POINTER(c.c_float), i32, vp, vp, vp, vp,
                                    vp, sz, vp]
    lib.cat_alpha_sweep.restype = c.c_int
    lib.cat_top1.argtypes = [vp, i64, i64, c.c_int, vp, vp]
    lib.cat_init_kmeanspp_workspace_bytes.argtypes = [i64, i32]
    lib.cat_init_kmeanspp_workspace_bytes.restype = sz
    lib.cat_init_kmeanspp.argtypes = [vp, i64, i64, i32, u64, c.c_int, vp, vp, vp, sz, vp]
    lib.cat_init_kmeanspp.restype = c.c_int
    lib.cat_top1.restype = c.c_int
    lib.cat_fit_restarts_workspace_bytes.argtypes = [i64, i64, i32, i32, c.c_int]
    lib.cat_fit_restarts_workspace_bytes.restype = sz
    lib.cat_fit_restarts.argtypes = [vp, vp, i64, i64, i32, i32, u64, i32, c.c_int, c.c_int, vp, vp, vp, vp, vp, vp, vp, vp,
                                     vp, sz, vp]
    lib.cat_fit_restarts.restype = c.c_int
    i32p = c.POINTER(c.c_int32)
    lib.cat_fit_multi_k_workspace_bytes.argtypes = [i64, i64, i32p, i32, i32, c.c_int]
    lib.cat_fit_multi_k_workspace_bytes.restype = sz
    lib.cat_fit_multi_k.argtypes = [vp, vp, i64, i64, i32p, i32, i32, u64, c.c_int, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.cat_fit_multi_k.restype = c.c_int
    lib.cat_fit_bounds_workspace_bytes.argtypes = [i64, i64, i32, i32, c.c_int]
    lib.cat_fit_bounds_workspace_bytes.restype = sz
    lib.cat_fit_bounds.argtypes = [vp, vp, i64, i64, i32, i32, u64, c.c_int, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.cat_fit_bounds.restype = c.c_int
    lib.cat_params_to_bf16.argtypes = [vp, i64, vp, vp]
    lib.cat_params_to_bf16.restype = c.c_int
    lib.cat_apply_lp_workspace_bytes.argtypes = [i64, i64, i32, c.c_int]
    lib.cat_apply_lp_workspace_bytes.restype = sz
    lib.cat_apply_lp.argtypes = [vp, i64, i64, i32, c.c_int, vp, vp, vp, c.c_float, c.c_int, vp, vp, vp, sz, vp]
    lib.cat_apply_lp.restype = c.c_int
    lib.cat_debug_multi_group_tiles.argtypes = [c.c_int]
    lib.cat_debug_multi_group_tiles.restype = c.c_int
    lib.cat_stream_probe.argtypes = [vp, vp, sz, vp]
    lib.cat_stream_probe.restype = c.c_int
    lib.cat_debug_padded_fit.argtypes = [c.c_int]
    lib.cat_debug_padded_fit.restype = c.c_int
    lib.cat_debug_apply_kernel.argtypes = [c.c_int]
    lib.cat_debug_apply_kernel.restype = c.c_int
    lib.cat_debug_list_capacity.argtypes = [c.c_int]
    lib.cat_debug_list_capacity.restype = c.c_int
    lib.cat_debug_rerank_queue.argtypes = [c.c_int]
    lib.cat_debug_rerank_queue.restype = c.c_int
    lib.cat_last_error.argtypes = []
    lib.cat_last_error.restype = c.c_char_p
    _lib = lib
    return lib


def _check(status):
    if status != 0:
        raise CatError(status, load_library().cat_last_error().decode())


def _dt(t):
    if t.dtype == torch.float32:
        return CAT_F32
    if t.dtype == torch.bfloat16:
        return CAT_BF16
    raise TypeError(f"lq/fp must be float32 or bfloat16, got {t.dtype}")


def _dev(t, dtype=None, shape=None, name="tensor"):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous device tensor")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} must have shape {tuple(shape)}, got {tuple(t.shape)}")
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def select_path(path):
    _check(load_library().cat_select_path(int(path)))


def allow_early_stop(on):
    """Let every Lloyd loop of the library leave out the passes after the partition has stopped changing (same outputs)."""
    _check(load_library().cat_allow_early_stop(1 if on else 0))


def debug_list_capacity(entries):
    """Test hook: capacity of the per-workgroup changed-row list of the fused Lloyd loop (0 = default)."""
    _check(load_library().cat_debug_list_capacity(int(entries)))


def debug_rerank_queue(entries):
    """Test hook: capacity of the per-workgroup queue of rows whose exact re-rank is put off (0 = default, -1 = no queue)."""
    _check(load_library().cat_debug_rerank_queue(int(entries)))


def debug_apply_kernel(which):
    """Test hook: 0 automatic, 1 never the row-tile inference kernel, 2 only the row-tile inference kernel."""
    _check(load_library().cat_debug_apply_kernel(int(which)))


def profile_enable(on):
    """Bracket every tile-kernel launch with HIP events on its stream (benchmarks only)."""
    _check(load_library().cat_profile_enable(1 if on else 0))


def profile_read():
    """Durations (ms) of the tile-kernel launches recorded since profile_enable(True)."""
    lib = load_library()
    n = lib.cat_profile_read(None, 0)
    if n < 0:
        raise CatError(4, "cat_profile_read failed")
    buf = (ctypes.c_float * max(n, 1))()
    lib.cat_profile_read(buf, n)
    return list(buf)[:n]


def cat_fit_workspace_bytes(N, D, K, dt=CAT_F32):
    return int(load_library().cat_fit_workspace_bytes(N, D, K, dt))


def cat_apply_workspace_bytes(N, D, K, dt=CAT_F32):
    return int(load_library().cat_apply_workspace_bytes(N, D, K, dt))


def _workspace(nbytes, device):
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def cat_init_indices(N, K, seed):
    """Host-side seeded row indices (list of K ints)."""
    buf = (ctypes.c_int64 * max(K, 1))()
    _check(load_library().cat_init_indices(N, K, seed & (2**64 - 1), buf))
    return list(buf)[:K]


def cat_fit(lq, fp, K, iters, seed=0, init_centroids=None, want_inertia=True, workspace=None, early_stop=False,
            bounds=False):
    """CAT Fitting on device tensors.  Returns a dict of device tensors:
    centroids, gamma, beta (K x D float32), assignments (N int32), counts (K int32),
    inertia (iters+1 float64, or None).  With ``early_stop`` (cat_fit_early_stop) the passes after the partition has
    stopped changing are not run, the outputs stay those of the full loop, and ``passes_skipped`` (1 int32) is added.
    With ``bounds`` (cat_fit_bounds) rows are left out of a pass by distance bounds, same outputs, and
    ``rows_evaluated`` (iters+1 int32) is added."""
    lib = load_library()
    N, D = lq.shape
    dt = _dt(lq)
    dev = lq.device
    if workspace is None:
        nbytes = (lib.cat_fit_bounds_workspace_bytes(N, D, K, iters, dt) if bounds
                  else lib.cat_fit_workspace_bytes(N, D, K, dt))
        workspace = _workspace(nbytes, dev)
    cent = torch.empty((K, D), dtype=torch.float32, device=dev)
    gamma = torch.empty((K, D), dtype=torch.float32, device=dev)
    beta = torch.empty((K, D), dtype=torch.float32, device=dev)
    a = torch.empty((N,), dtype=torch.int32, device=dev)
    counts = torch.empty((K,), dtype=torch.int32, device=dev)
    inertia = torch.empty((max(iters, 0) + 1,), dtype=torch.float64, device=dev) if want_inertia else None
    head = (_dev(lq, name="lq"), _dev(fp, lq.dtype, (N, D), "fp"), N, D, K, iters,
            seed & (2**64 - 1), dt, _dev(init_centroids, torch.float32, (K, D), "init_centroids"),
            cent.data_ptr(), gamma.data_ptr(), beta.data_ptr(), a.data_ptr(), counts.data_ptr(),
            None if inertia is None else inertia.data_ptr())
    tail = (workspace.data_ptr(), workspace.numel(), _stream())
    res = dict(centroids=cent, gamma=gamma, beta=beta, assignments=a, counts=counts, inertia=inertia)
    if bounds:
        res["rows_evaluated"] = torch.empty((max(iters, 0) + 1,), dtype=torch.int32, device=dev)
        _check(lib.cat_fit_bounds(*head, res["rows_evaluated"].data_ptr(), *tail))
    elif early_stop:
        res["passes_skipped"] = torch.empty((1,), dtype=torch.int32, device=dev)
        _check(lib.cat_fit_early_stop(*head, res["passes_skipped"].data_ptr(), *tail))
    else:
        _check(lib.cat_fit(*head, *tail))
    return res


def cat_apply(lq, centroids, gamma, beta, alpha=1.0, want_assignments=True, out=None, workspace=None):
    """CAT Inferencing.  Returns (corrected, assignments or None)."""
    lib = load_library()
    N, D = lq.shape
    K = centroids.shape[0]
    dt = _dt(lq)
    dev = lq.device
    if workspace is None:
        workspace = _workspace(lib.cat_apply_workspace_bytes(N, D, K, dt), dev)
    if out is None:
        out = torch.empty_like(lq)
    a = torch.empty((N,), dtype=torch.int32, device=dev) if want_assignments else None
    _check(lib.cat_apply(_dev(lq, name="lq"), N, D, K, dt, _dev(centroids, torch.float32, (K, D), "centroids"),
                         _dev(gamma, torch.float32, (K, D), "gamma"), _dev(beta, torch.float32, (K, D), "beta"),
                         float(alpha), _dev(out, lq.dtype, (N, D), "out"),
                         None if a is None else a.data_ptr(),
                         workspace.data_ptr(), workspace.numel(), _stream()))
    return out, a


def cat_apply_static(lq, centroids, gamma, beta, alpha=1.0, out=None, assignments=None):
    """cat_apply without a workspace (the library's built-in scratch array).  The library call allocates nothing;
    pass ``out`` (and ``assignments``, or leave it None to skip them) to keep this wrapper from allocating too.
    Returns (corrected, assignments or None)."""
    lib = load_library()
    N, D = lq.shape
    K = centroids.shape[0]
    dt = _dt(lq)
    if out is None:
        out = torch.empty_like(lq)
    _check(lib.cat_apply_static(_dev(lq, name="lq"), N, D, K, dt, _dev(centroids, torch.float32, (K, D), "centroids"),
                                _dev(gamma, torch.float32, (K, D), "gamma"), _dev(beta, torch.float32, (K, D), "beta"),
                                float(alpha), _dev(out, lq.dtype, (N, D), "out"),
                                _dev(assignments, torch.int32, (N,), "assignments"), _stream()))
    return out, assignments


def cat_assign(lq, centroids, workspace=None):
    """Assignment step.  Returns (assignments int32 N, counts int32 K, inertia float64 [1])."""
    lib = load_library()
    N, D = lq.shape
    K = centroids.shape[0]
    dt = _dt(lq)
    dev = lq.device
    if workspace is None:
        workspace = _workspace(lib.cat_fit_workspace_bytes(N, D, K, dt), dev)
    a = torch.empty((N,), dtype=torch.int32, device=dev)
    counts = torch.empty((K,), dtype=torch.int32, device=dev)
    inertia = torch.empty((1,), dtype=torch.float64, device=dev)
    _check(lib.cat_assign(_dev(lq, name="lq"), N, D, K, dt, _dev(centroids, torch.float32, (K, D), "centroids"),
                          a.data_ptr(), counts.data_ptr(), inertia.data_ptr(),
                          workspace.data_ptr(), workspace.numel(), _stream()))
    return a, counts, inertia


def cat_update(lq, assignments, prev_centroids, workspace=None):
    """Centroid update step.  Returns (centroids float32 K x D, counts int32 K)."""
    lib = load_library()
    N, D = lq.shape
    K = prev_centroids.shape[0]
    dt = _dt(lq)
    dev = lq.device
    if workspace is None:
        workspace = _workspace(lib.cat_fit_workspace_bytes(N, D, K, dt), dev)
    cent = torch.empty((K, D), dtype=torch.float32, device=dev)
    counts = torch.empty((K,), dtype=torch.int32, device=dev)
    _check(lib.cat_update(_dev(lq, name="lq"), _dev(assignments, torch.int32, (N,), "assignments"), N, D, K, dt,
                          _dev(prev_centroids, torch.float32, (K, D), "prev_centroids"),
                          cent.data_ptr(), counts.data_ptr(),
                          workspace.data_ptr(), workspace.numel(), _stream()))
    return cent, counts


def cat_stats(lq, fp, assignments, K, centroids=None, workspace=None):
    """Per-cluster affine fit for a given partition.  Returns (gamma, beta, counts)."""
    lib = load_library()
    N, D = lq.shape
    dt = _dt(lq)
    dev = lq.device
    if workspace is None:
        workspace = _workspace(lib.cat_fit_workspace_bytes(N, D, K, dt), dev)
    gamma = torch.empty((K, D), dtype=torch.float32, device=dev)
    beta = torch.empty((K, D), dtype=torch.float32, device=dev)
    counts = torch.empty((K,), dtype=torch.int32, device=dev)
    _check(lib.cat_stats(_dev(lq, name="lq"), _dev(fp, lq.dtype, (N, D), "fp"),
                         _dev(assignments, torch.int32, (N,), "assignments"), N, D, K, dt,
                         _dev(centroids, torch.float32, (K, D), "centroids"),
                         gamma.data_ptr(), beta.data_ptr(), counts.data_ptr(),
                         workspace.data_ptr(), workspace.numel(), _stream()))
    return gamma, beta, counts


def cat_pca_fit(lq, p, sweeps=0, workspace=None):
    """PCA front-end: returns (mean D float32, components p x D float32, eigenvalues p float64), device tensors."""
    lib = load_library()
    N, D = lq.shape
    dt = _dt(lq)
    dev = lq.device
    if workspace is None:
        workspace = _workspace(lib.cat_pca_workspace_bytes(N, D, p, dt), dev)
    mean = torch.empty((D,), dtype=torch.float32, device=dev)
    comps = torch.empty((p, D), dtype=torch.float32, device=dev)
    evals = torch.empty((p,), dtype=torch.float64, device=dev)
    _check(lib.cat_pca_fit(_dev(lq, name="lq"), N, D, p, dt, sweeps, mean.data_ptr(), comps.data_ptr(), evals.data_ptr(),
                           workspace.data_ptr(), workspace.numel(), _stream()))
    return mean, comps, evals


def cat_pca_project(lq, mean, components):
    """z = (lq - mean) @ components.T as float32 N x p."""
    lib = load_library()
    N, D = lq.shape
    p = components.shape[0]
    z = torch.empty((N, p), dtype=torch.float32, device=lq.device)
    _check(lib.cat_pca_project(_dev(lq, name="lq"), N, D, p, _dt(lq), _dev(mean, torch.float32, (D,), "mean"),
                               _dev(components, torch.float32, (p, D), "components"), z.data_ptr(), _stream()))
    return z


def cat_apply_assigned(lq, assignments, gamma, beta, alpha=1.0, out=None):
    """Affine correction by given labels (the inference step when clusters are found in PCA space)."""
    lib = load_library()
    N, D = lq.shape
    K = gamma.shape[0]
    if out is None:
        out = torch.empty_like(lq)
    _check(lib.cat_apply_assigned(_dev(lq, name="lq"), _dev(assignments, torch.int32, (N,), "assignments"), N, D, K, _dt(lq),
                                  _dev(gamma, torch.float32, (K, D), "gamma"), _dev(beta, torch.float32, (K, D), "beta"),
                                  float(alpha), _dev(out, lq.dtype, (N, D), "out"), _stream()))
    return out


def cat_alpha_sweep(lq, assignments, gamma, beta, alphas, fp=None, labels=None, want_top1=False, workspace=None):
    """One fitted transformation evaluated at every alpha of a list in one pass over the rows (the ablation on
    the blending coefficient).  Returns a dict of device tensors: ``hits`` (n int64; with labels), ``sq_err``
    (n float64) and ``moments`` (3 float64; with fp), ``top1`` (N x n int32; with want_top1)."""
    lib = load_library()
    N, D = lq.shape
    K = gamma.shape[0]
    dev = lq.device
    al = [float(a) for a in alphas]
    n = len(al)
    arr = (ctypes.c_float * max(n, 1))(*al)
    if workspace is None:
        workspace = _workspace(lib.cat_alpha_sweep_workspace_bytes(), dev)
    hits = torch.empty((n,), dtype=torch.int64, device=dev) if labels is not None else None
    sq = torch.empty((n,), dtype=torch.float64, device=dev) if fp is not None else None
    mom = torch.empty((3,), dtype=torch.float64, device=dev) if fp is not None else None
    top1 = torch.empty((N, n), dtype=torch.int32, device=dev) if want_top1 else None
    _check(lib.cat_alpha_sweep(_dev(lq, name="lq"), _dev(fp, lq.dtype, (N, D), "fp"), _dev(labels, torch.int32, (N,), "labels"),
                               _dev(assignments, torch.int32, (N,), "assignments"), N, D, K, _dt(lq),
                               _dev(gamma, torch.float32, (K, D), "gamma"), _dev(beta, torch.float32, (K, D), "beta"),
                               arr, n, _dev(hits), _dev(sq), _dev(mom), _dev(top1),
                               workspace.data_ptr(), workspace.numel(), _stream()))
    return dict(hits=hits, sq_err=sq, moments=mom, top1=top1)


def cat_top1(x, out=None):
    """Position of the largest entry of every row (first on ties): N int32."""
    lib = load_library()
    N, D = x.shape
    if out is None:
        out = torch.empty((N,), dtype=torch.int32, device=x.device)
    _check(lib.cat_top1(_dev(x, name="x"), N, D, _dt(x), _dev(out, torch.int32, (N,), "out"), _stream()))
    return out


def cat_init_kmeanspp(lq, K, seed=0, workspace=None):
    """D^2-weighted seeding (k-means++).  Returns (centroids K x D float32, row indices K int64), device tensors;
    pass the centroids to ``cat_fit(..., init_centroids=...)``."""
    lib = load_library()
    N, D = lq.shape
    if workspace is None:
        workspace = _workspace(lib.cat_init_kmeanspp_workspace_bytes(N, K), lq.device)
    cent = torch.empty((K, D), dtype=torch.float32, device=lq.device)
    idx = torch.empty((K,), dtype=torch.int64, device=lq.device)
    _check(lib.cat_init_kmeanspp(_dev(lq, name="lq"), N, D, K, seed & (2**64 - 1), _dt(lq), cent.data_ptr(), idx.data_ptr(),
                                 workspace.data_ptr(), workspace.numel(), _stream()))
    return cent, idx


CAT_SEED_ROWS, CAT_SEED_KMEANSPP = 0, 1


def cat_fit_restarts(lq, fp, K, iters, seed=0, restarts=4, seeding=CAT_SEED_ROWS, workspace=None):
    """``restarts`` runs of the clustering (run r seeded with ``seed + r``), the one with the lowest final objective
    kept, then the affine fit on its partition.  Returns the dict of ``cat_fit`` plus ``best_run`` (1 int32) and
    ``final_inertia`` (restarts float64), all device tensors."""
    lib = load_library()
    N, D = lq.shape
    dt = _dt(lq)
    dev = lq.device
    if workspace is None:
        workspace = _workspace(lib.cat_fit_restarts_workspace_bytes(N, D, K, iters, dt), dev)
    f32 = dict(dtype=torch.float32, device=dev)
    cent, gamma, beta = torch.empty((K, D), **f32), torch.empty((K, D), **f32), torch.empty((K, D), **f32)
    a = torch.empty((N,), dtype=torch.int32, device=dev)
    counts = torch.empty((K,), dtype=torch.int32, device=dev)
    inertia = torch.empty((max(iters, 0) + 1,), dtype=torch.float64, device=dev)
    best = torch.empty((1,), dtype=torch.int32, device=dev)
    finals = torch.empty((max(restarts, 1),), dtype=torch.float64, device=dev)
    _check(lib.cat_fit_restarts(_dev(lq, name="lq"), _dev(fp, lq.dtype, (N, D), "fp"), N, D, K, iters, seed & (2**64 - 1),
                                restarts, int(seeding), dt, cent.data_ptr(), gamma.data_ptr(), beta.data_ptr(), a.data_ptr(),
                                counts.data_ptr(), inertia.data_ptr(), best.data_ptr(), finals.data_ptr(),
                                workspace.data_ptr(), workspace.numel(), _stream()))
    return dict(centroids=cent, gamma=gamma, beta=beta, assignments=a, counts=counts, inertia=inertia, best_run=best,
                final_inertia=finals)


def stream_probe(src, dst=None):
    """One launch that only reads ``src`` (``dst`` None) or copies it to ``dst``: what the memory system gives (cat_stream_probe)."""
    nbytes = src.numel() * src.element_size()
    if dst is not None and dst.numel() * dst.element_size() != nbytes:
        raise ValueError("dst must have the size of src")
    _check(load_library().cat_stream_probe(src.data_ptr(), None if dst is None else dst.data_ptr(), nbytes, _stream()))


def debug_padded_fit(on):
    """False keeps fits of rows that are not whole 16-byte groups on the streaming kernels (default: a padded copy)."""
    _check(load_library().cat_debug_padded_fit(int(bool(on))))


def debug_multi_group_tiles(tiles):
    """At most ``tiles`` 16-cluster tiles per group of ``cat_fit_multi_k`` (1 runs every entry on its own)."""
    _check(load_library().cat_debug_multi_group_tiles(int(tiles)))


def cat_fit_multi_k(lq, fp, Ks, iters, seed=0, want_inertia=True, workspace=None):
    """CAT Fitting for every cluster count in ``Ks`` (cat_fit_multi_k): the fits share the reads of the rows where the
    shape allows it.  Returns a list of dicts like ``cat_fit``'s, one per entry of ``Ks``; their tensors are views of the
    concatenated outputs of the call."""
    lib = load_library()
    N, D = lq.shape
    dt = _dt(lq)
    dev = lq.device
    Ks = [int(k) for k in Ks]
    nK = len(Ks)
    ks = (ctypes.c_int32 * max(nK, 1))(*Ks)
    if workspace is None:
        workspace = _workspace(lib.cat_fit_multi_k_workspace_bytes(N, D, ks, nK, iters, dt), dev)
    tot = sum(Ks)
    f32 = dict(dtype=torch.float32, device=dev)
    cent, gamma, beta = torch.empty((tot, D), **f32), torch.empty((tot, D), **f32), torch.empty((tot, D), **f32)
    a = torch.empty((nK, N), dtype=torch.int32, device=dev)
    counts = torch.empty((tot,), dtype=torch.int32, device=dev)
    inertia = torch.empty((nK, max(iters, 0) + 1), dtype=torch.float64, device=dev) if want_inertia else None
    _check(lib.cat_fit_multi_k(_dev(lq, name="lq"), _dev(fp, lq.dtype, (N, D), "fp"), N, D, ks, nK, iters, seed & (2**64 - 1), dt,
                               cent.data_ptr(), gamma.data_ptr(), beta.data_ptr(), a.data_ptr(), counts.data_ptr(),
                               None if inertia is None else inertia.data_ptr(), workspace.data_ptr(), workspace.numel(),
                               _stream()))
    out, r = [], 0
    for i, K in enumerate(Ks):
        out.append(dict(centroids=cent[r:r + K], gamma=gamma[r:r + K], beta=beta[r:r + K], assignments=a[i],
                        counts=counts[r:r + K], inertia=None if inertia is None else inertia[i]))
        r += K
    return out


def cat_params_to_bf16(x):
    """The bfloat16 values nearest to a float32 device tensor (cat_params_to_bf16), as a torch.bfloat16 tensor."""
    x = x.contiguous()
    out = torch.empty(x.shape, dtype=torch.bfloat16, device=x.device)
    _check(load_library().cat_params_to_bf16(_dev(x, torch.float32, name="x"), x.numel(), out.data_ptr(), _stream()))
    return out


def cat_apply_lp(lq, centroids, gamma, beta, alpha=1.0, bf16_out=True, want_assignments=True, out=None, workspace=None):
    """CAT Inferencing with parameters stored as bfloat16 tensors (cat_apply_lp).  ``bf16_out``: the corrected rows of
    float32 inputs are written as bfloat16.  Returns (corrected, assignments or None)."""
    lib = load_library()
    N, D = lq.shape
    K = centroids.shape[0]
    dt = _dt(lq)
    dev = lq.device
    out_dt = CAT_BF16 if (bf16_out or dt == CAT_BF16) else CAT_F32
    if workspace is None:
        workspace = _workspace(lib.cat_apply_lp_workspace_bytes(N, D, K, dt), dev)
    if out is None:
        out = torch.empty((N, D), dtype=torch.bfloat16 if out_dt == CAT_BF16 else torch.float32, device=dev)
    a = torch.empty((N,), dtype=torch.int32, device=dev) if want_assignments else None
    _check(lib.cat_apply_lp(_dev(lq, name="lq"), N, D, K, dt, _dev(centroids, torch.bfloat16, (K, D), "centroids"),
                            _dev(gamma, torch.bfloat16, (K, D), "gamma"), _dev(beta, torch.bfloat16, (K, D), "beta"),
                            float(alpha), out_dt, out.data_ptr(), None if a is None else a.data_ptr(),
                            workspace.data_ptr(), workspace.numel(), _stream()))
    return out, a


def cat_fit_pca(lq, fp, K, p, iters, seed=0, want_inertia=True, workspace=None):
    """CAT Fitting with the PCA front-end (clusters from the p leading principal components).  Returns a dict:
    mean, components, centroids_z (K x p), gamma, beta (K x D), assignments, counts, inertia."""
    lib = load_library()
    N, D = lq.shape
    dt = _dt(lq)
    dev = lq.device
    if workspace is None:
        workspace = _workspace(lib.cat_fit_pca_workspace_bytes(N, D, K, p, dt), dev)
    f32 = dict(dtype=torch.float32, device=dev)
    mean, comps = torch.empty((D,), **f32), torch.empty((p, D), **f32)
    cz, gamma, beta = torch.empty((K, p), **f32), torch.empty((K, D), **f32), torch.empty((K, D), **f32)
    a = torch.empty((N,), dtype=torch.int32, device=dev)
    counts = torch.empty((K,), dtype=torch.int32, device=dev)
    inertia = torch.empty((max(iters, 0) + 1,), dtype=torch.float64, device=dev) if want_inertia else None
    _check(lib.cat_fit_pca(_dev(lq, name="lq"), _dev(fp, lq.dtype, (N, D), "fp"), N, D, K, p, iters, seed & (2**64 - 1), dt,
                           mean.data_ptr(), comps.data_ptr(), cz.data_ptr(), gamma.data_ptr(), beta.data_ptr(), a.data_ptr(),
                           counts.data_ptr(), None if inertia is None else inertia.data_ptr(),
                           workspace.data_ptr(), workspace.numel(), _stream()))
    return dict(mean=mean, components=comps, centroids_z=cz, gamma=gamma, beta=beta, assignments=a, counts=counts,
                inertia=inertia)


def cat_apply_pca(lq, mean, components, centroids_z, gamma, beta, alpha=1.0, want_assignments=True, out=None, workspace=None):
    """CAT Inferencing with the PCA front-end.  Returns (corrected, assignments or None)."""
    lib = load_library()
    N, D = lq.shape
    K, p = centroids_z.shape
    dt = _dt(lq)
    dev = lq.device
    if workspace is None:
        workspace = _workspace(lib.cat_apply_pca_workspace_bytes(N, D, K, p, dt), dev)
    if out is None:
        out = torch.empty_like(lq)
    a = torch.empty((N,), dtype=torch.int32, device=dev) if want_assignments else None
    _check(lib.cat_apply_pca(_dev(lq, name="lq"), N, D, K, p, dt, _dev(mean, torch.float32, (D,), "mean"),
                             _dev(components, torch.float32, (p, D), "components"),
                             _dev(centroids_z, torch.float32, (K, p), "centroids_z"),
                             _dev(gamma, torch.float32, (K, D), "gamma"), _dev(beta, torch.float32, (K, D), "beta"),
                             float(alpha), _dev(out, lq.dtype, (N, D), "out"), None if a is None else a.data_ptr(),
                             workspace.data_ptr(), workspace.numel(), _stream()))
    return out, a
