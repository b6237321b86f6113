"""ctypes binding of the C oracle (``cat_oracle.c``).

Test infrastructure only.  Arrays go in as contiguous numpy float32 (inputs) and
float64 (centroids, gamma, beta); every result is float64 / int32 / int64.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "cat_oracle.c")
_SO = os.path.join(_HERE, "libcat_oracle.so")
_lib = None


def build(force=False):
    """Compile the oracle with gcc (-O2, no fast-math).  Returns the .so path."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
               "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _SO


def _load():
    global _lib
    if _lib is not None:
        return _lib
    lib = ctypes.CDLL(build())
    c = ctypes
    f32p, f64p = c.POINTER(c.c_float), c.POINTER(c.c_double)
    i32p, i64p = c.POINTER(c.c_int32), c.POINTER(c.c_int64)
    lib.cat_oracle_threads.restype = c.c_int
    lib.cat_oracle_splitmix64.restype = c.c_uint64
    lib.cat_oracle_splitmix64.argtypes = [c.c_uint64, c.c_uint64]
    lib.cat_oracle_init_indices.argtypes = [c.c_int64, c.c_int32, c.c_uint64, i64p]
    lib.cat_oracle_assign.argtypes = [f32p, c.c_int64, c.c_int64, c.c_int32, f64p, i32p, f64p, f64p]
    lib.cat_oracle_distances.argtypes = [f32p, c.c_int64, c.c_int64, c.c_int32, f64p, f64p]
    lib.cat_oracle_update.argtypes = [f32p, i32p, c.c_int64, c.c_int64, c.c_int32, f64p, i64p]
    lib.cat_oracle_affine.argtypes = [f32p, f32p, i32p, c.c_int64, c.c_int64, c.c_int32, f64p, f64p, i64p]
    lib.cat_oracle_fit.argtypes = [f32p, f32p, c.c_int64, c.c_int64, c.c_int32, c.c_int32, c.c_uint64,
                                   f64p, f64p, f64p, f64p, i32p, i64p, f64p]
    lib.cat_oracle_apply.argtypes = [f32p, c.c_int64, c.c_int64, c.c_int32, f64p, f64p, f64p,
                                     c.c_double, f64p, i32p]
    lib.cat_oracle_colmean.argtypes = [f32p, c.c_int64, c.c_int64, f64p]
    lib.cat_oracle_covariance.argtypes = [f32p, c.c_int64, c.c_int64, f64p, f64p]
    lib.cat_oracle_project.argtypes = [f32p, c.c_int64, c.c_int64, c.c_int32, f64p, f64p, f64p]
    lib.cat_oracle_alpha_sweep.argtypes = [f32p, f32p, i32p, i32p, c.c_int64, c.c_int64, c.c_int32, f64p, f64p,
                                           f64p, c.c_int32, i64p, f64p, i32p, f64p]
    lib.cat_oracle_kmeanspp.argtypes = [f32p, c.c_int64, c.c_int64, c.c_int32, c.c_uint64, i64p]
    for fn in ("cat_oracle_colmean", "cat_oracle_covariance", "cat_oracle_project", "cat_oracle_alpha_sweep",
               "cat_oracle_kmeanspp"):
        getattr(lib, fn).restype = None
    for fn in ("cat_oracle_init_indices", "cat_oracle_assign", "cat_oracle_distances", "cat_oracle_update",
               "cat_oracle_affine", "cat_oracle_fit", "cat_oracle_apply"):
        getattr(lib, fn).restype = None
    _lib = lib
    return lib


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _f64(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _p(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


def threads():
    return int(_load().cat_oracle_threads())


def splitmix64(seed, t):
    return int(_load().cat_oracle_splitmix64(seed & (2**64 - 1), t))


def init_indices(N, K, seed):
    idx = np.empty(K, dtype=np.int64)
    _load().cat_oracle_init_indices(N, K, seed & (2**64 - 1), _p(idx, ctypes.c_int64))
    return idx


def assign(lq, centroids, want_distances=False):
    """Nearest centroid per row (lowest index on ties).  Returns a, or (a, d1, d2)."""
    lq, plq = _f32(lq)
    cent, pc = _f64(centroids)
    N, D = lq.shape
    K = cent.shape[0]
    assert cent.shape == (K, D)
    a = np.empty(N, dtype=np.int32)
    if want_distances:
        d1 = np.empty(N, dtype=np.float64)
        d2 = np.empty(N, dtype=np.float64)
        _load().cat_oracle_assign(plq, N, D, K, pc, _p(a, ctypes.c_int32),
                                  _p(d1, ctypes.c_double), _p(d2, ctypes.c_double))
        return a, d1, d2
    _load().cat_oracle_assign(plq, N, D, K, pc, _p(a, ctypes.c_int32), None, None)
    return a


def distances(lq, centroids):
    lq, plq = _f32(lq)
    cent, pc = _f64(centroids)
    N, D = lq.shape
    K = cent.shape[0]
    out = np.empty((N, K), dtype=np.float64)
    _load().cat_oracle_distances(plq, N, D, K, pc, _p(out, ctypes.c_double))
    return out


def update(lq, assignments, centroids):
    """One centroid update; returns (new_centroids, counts)."""
    lq, plq = _f32(lq)
    a, pa = _i32(assignments)
    cent = np.array(centroids, dtype=np.float64, order="C", copy=True)
    N, D = lq.shape
    K = cent.shape[0]
    assert a.min() >= 0 and a.max() < K
    counts = np.empty(K, dtype=np.int64)
    _load().cat_oracle_update(plq, pa, N, D, K, _p(cent, ctypes.c_double), _p(counts, ctypes.c_int64))
    return cent, counts


def affine(lq, fp, assignments, K):
    """Per-cluster per-channel gamma, beta; returns (gamma, beta, counts)."""
    lq, plq = _f32(lq)
    fp, pfp = _f32(fp)
    a, pa = _i32(assignments)
    N, D = lq.shape
    assert fp.shape == (N, D)
    assert a.min() >= 0 and a.max() < K
    gamma = np.empty((K, D), dtype=np.float64)
    beta = np.empty((K, D), dtype=np.float64)
    counts = np.empty(K, dtype=np.int64)
    _load().cat_oracle_affine(plq, pfp, pa, N, D, K, _p(gamma, ctypes.c_double),
                              _p(beta, ctypes.c_double), _p(counts, ctypes.c_int64))
    return gamma, beta, counts


def fit(lq, fp, K, iters, seed=0, init_centroids=None):
    """CAT Fitting.  Returns dict(centroids, gamma, beta, assignments, counts, inertia)."""
    lq, plq = _f32(lq)
    fp, pfp = _f32(fp)
    N, D = lq.shape
    assert fp.shape == (N, D) and 1 <= K <= N and iters >= 0
    cent = np.empty((K, D), dtype=np.float64)
    gamma = np.empty((K, D), dtype=np.float64)
    beta = np.empty((K, D), dtype=np.float64)
    a = np.empty(N, dtype=np.int32)
    counts = np.empty(K, dtype=np.int64)
    inertia = np.empty(iters + 1, dtype=np.float64)
    if init_centroids is not None:
        init, pinit = _f64(init_centroids)
        assert init.shape == (K, D)
    else:
        pinit = None
    _load().cat_oracle_fit(plq, pfp, N, D, K, iters, seed & (2**64 - 1), pinit,
                           _p(cent, ctypes.c_double), _p(gamma, ctypes.c_double), _p(beta, ctypes.c_double),
                           _p(a, ctypes.c_int32), _p(counts, ctypes.c_int64), _p(inertia, ctypes.c_double))
    return dict(centroids=cent, gamma=gamma, beta=beta, assignments=a, counts=counts, inertia=inertia)


def apply(lq, centroids, gamma, beta, alpha=1.0):
    """CAT Inferencing.  Returns (corrected float64 N x D, assignments)."""
    lq, plq = _f32(lq)
    cent, pc = _f64(centroids)
    g, pg = _f64(gamma)
    b, pb = _f64(beta)
    N, D = lq.shape
    K = cent.shape[0]
    assert cent.shape == (K, D) and g.shape == (K, D) and b.shape == (K, D)
    out = np.empty((N, D), dtype=np.float64)
    a = np.empty(N, dtype=np.int32)
    _load().cat_oracle_apply(plq, N, D, K, pc, pg, pb, float(alpha), _p(out, ctypes.c_double),
                             _p(a, ctypes.c_int32))
    return out, a


# ---------------------------------------------------------------------------
# PCA front-end (Sec. 3.1; Alg. 1 / Alg. 2, first step)
# ---------------------------------------------------------------------------
def covariance(lq):
    """Column means (D) and the population covariance (D x D) of the rows, in double."""
    lib = _load()
    x, xp = _f32(lq)
    N, D = x.shape
    mean = np.empty(D, dtype=np.float64)
    cov = np.empty((D, D), dtype=np.float64)
    lib.cat_oracle_colmean(xp, N, D, _p(mean, ctypes.c_double))
    lib.cat_oracle_covariance(xp, N, D, _p(mean, ctypes.c_double), _p(cov, ctypes.c_double))
    return mean, cov


def pca_fit(lq, p):
    """The p leading principal directions of the rows of ``lq``.

    Returns (mean D, components p x D, eigenvalues p): eigenvalues of the population covariance in
    descending order (equal eigenvalues keep the order of the library routine, reversed), each
    direction a unit vector whose entry of largest magnitude (the first such entry) is positive.
    The symmetric eigendecomposition is numpy.linalg.eigh (LAPACK)."""
    mean, cov = covariance(lq)
    w, v = np.linalg.eigh(cov)  # ascending
    order = np.arange(len(w))[::-1][:p]
    evals = w[order].copy()
    comps = v[:, order].T.copy()
    for c in range(comps.shape[0]):
        j = int(np.argmax(np.abs(comps[c])))
        if comps[c, j] < 0:
            comps[c] = -comps[c]
    return mean, comps, evals


def pca_project(lq, mean, comps):
    """(lq - mean) @ comps.T in double: N x p."""
    lib = _load()
    x, xp = _f32(lq)
    N, D = x.shape
    m = np.ascontiguousarray(mean, dtype=np.float64)
    w = np.ascontiguousarray(comps, dtype=np.float64)
    pdim = w.shape[0]
    z = np.empty((N, pdim), dtype=np.float64)
    lib.cat_oracle_project(xp, N, D, pdim, _p(m, ctypes.c_double), _p(w, ctypes.c_double), _p(z, ctypes.c_double))
    return z


# ---------------------------------------------------------------------------
# Sweep of the blending coefficient (Sec. 3.1 alpha display; ablation on alpha, Sec. 5)
# ---------------------------------------------------------------------------
def alpha_sweep(lq, assignments, gamma, beta, alphas, fp=None, labels=None):
    """One fitted transformation evaluated at every alpha of a list, rows labelled by ``assignments``.

    Returns a dict: ``top1`` (N x n int32, position of the largest corrected entry, first on ties),
    ``margin`` (N x n, largest minus second largest corrected entry), ``hits`` (n int64, rows whose
    top1 equals ``labels``; zeros without labels) and ``sq_err`` (n, summed squared difference to
    ``fp``; zeros without fp)."""
    lib = _load()
    x, xp = _f32(lq)
    N, D = x.shape
    g, pg = _f64(gamma)
    b, pb = _f64(beta)
    K = g.shape[0]
    assert g.shape == (K, D) and b.shape == (K, D)
    a = np.ascontiguousarray(assignments, dtype=np.int32)
    assert a.shape == (N,)
    al = np.ascontiguousarray(alphas, dtype=np.float64)
    n = al.shape[0]
    null_f = ctypes.POINTER(ctypes.c_float)()
    null_i = ctypes.POINTER(ctypes.c_int32)()
    if fp is not None:
        y, yp = _f32(fp)
        assert y.shape == (N, D)
    else:
        yp = null_f
    if labels is not None:
        lab = np.ascontiguousarray(labels, dtype=np.int32)
        assert lab.shape == (N,)
        lp = _p(lab, ctypes.c_int32)
    else:
        lp = null_i
    hits = np.zeros(n, dtype=np.int64)
    sq = np.zeros(n, dtype=np.float64)
    top1 = np.empty((N, n), dtype=np.int32)
    margin = np.empty((N, n), dtype=np.float64)
    lib.cat_oracle_alpha_sweep(xp, yp, lp, _p(a, ctypes.c_int32), N, D, K, pg, pb, _p(al, ctypes.c_double), n,
                               _p(hits, ctypes.c_int64), _p(sq, ctypes.c_double), _p(top1, ctypes.c_int32),
                               _p(margin, ctypes.c_double))
    return dict(top1=top1, margin=margin, hits=hits, sq_err=sq)


# ---------------------------------------------------------------------------
# D^2-weighted seeding (k-means++, Arthur and Vassilvitskii 2007)
# ---------------------------------------------------------------------------
def kmeanspp(lq, K, seed=0):
    """K row indices (int64, in the order drawn): the first uniform, each further one with probability
    proportional to the squared distance to the nearest row chosen so far."""
    x, xp = _f32(lq)
    N, D = x.shape
    assert 1 <= K <= N
    idx = np.empty(K, dtype=np.int64)
    _load().cat_oracle_kmeanspp(xp, N, D, K, seed & (2**64 - 1), _p(idx, ctypes.c_int64))
    return idx


# ---------------------------------------------------------------------------
# Several runs, the best kept
# ---------------------------------------------------------------------------
def fit_restarts(lq, fp, K, iters, seed=0, restarts=4, kmeanspp_seeding=False):
    """``restarts`` runs of ``fit`` (run r seeded with ``seed + r``; the D^2-weighted rows of ``kmeanspp`` as initial
    centroids if asked), the run with the lowest final objective kept, the first one on ties.  Returns the dict of
    the kept run plus ``best_run`` and ``final_inertia`` (the final objective of every run)."""
    best, finals = None, []
    for r in range(restarts):
        init = None
        if kmeanspp_seeding:
            init = np.asarray(lq, dtype=np.float32)[kmeanspp(lq, K, seed=seed + r)].astype(np.float64)
        run = fit(lq, fp, K, iters, seed=seed + r, init_centroids=init)
        finals.append(float(run["inertia"][-1]))
        if best is None or finals[-1] < best["inertia"][-1]:
            best = dict(run, best_run=r)
    best["final_inertia"] = np.asarray(finals)
    return best


def fit_early_stop(lq, fp, K, iters, seed=0, init_centroids=None):
    """``fit`` with the Lloyd loop left at the first pass whose assignments repeat those of the pass before
    (the partition is then a fixed point of the iteration: the means, hence every later pass, cannot change).

    Written as the sequence of the oracle's own steps: assign, compare with the previous assignments, update.
    The objective of the passes that are not run is the one of the last pass that was.  Returns the dict of
    ``fit`` plus ``stable_at``: the index t >= 1 of the first repeating pass, or -1 if none of the iters + 1
    passes repeats its predecessor."""
    x = np.ascontiguousarray(lq, dtype=np.float32)
    N, D = x.shape
    if init_centroids is None:
        cent = x[init_indices(N, K, seed)].astype(np.float64)
    else:
        cent = np.array(init_centroids, dtype=np.float64)
    inertia = np.empty(iters + 1, dtype=np.float64)
    prev, stable_at = None, -1
    for t in range(iters + 1):
        a, d1, _ = assign(x, cent, want_distances=True)
        inertia[t] = d1.sum()
        if prev is not None and (a == prev).all():
            stable_at = t
            inertia[t:] = inertia[t]
            break
        if t < iters:
            cent, _ = update(x, a, cent)
            prev = a
    gamma, beta, counts = affine(x, fp, a, K)
    return dict(centroids=cent, gamma=gamma, beta=beta, assignments=a, counts=counts, inertia=inertia,
                stable_at=stable_at)


# ---------------------------------------------------------------------------
# Fits for several cluster counts (the paper's ablation on the number of clusters, Sec. 5 and its appendix,
# sweeps a grid of K at fixed PCA dimension and blending coefficient)
# ---------------------------------------------------------------------------
def fit_multi_k(lq, fp, Ks, iters, seed=0):
    """One independent ``fit`` per cluster count in ``Ks``, each seeded with ``seed``.  Returns the list of
    their dicts, in the order of ``Ks``.  (Sharing the reads of the rows between the fits is an implementation
    matter: it changes nothing that is computed.)"""
    return [fit(lq, fp, int(K), iters, seed=seed) for K in Ks]


# ---------------------------------------------------------------------------
# Low-precision deployment (Sec. 3.1 remarks that the clustering yields low-precision gamma, beta; the paper
# gives no mechanism): parameters stored as bfloat16, inference output stored as bfloat16
# ---------------------------------------------------------------------------
def to_bf16(x):
    """The bfloat16 value nearest to each entry of ``x`` (8 significant bits, ties to the even significand),
    returned as float64.  From the definition: x = m * 2^e with 1/2 <= |m| < 1, so the spacing of bfloat16 numbers
    around x is 2^(e - 8).  Exponent range is not modelled (no overflow / subnormal handling): finite inputs of
    ordinary size only."""
    x = np.asarray(x, dtype=np.float64)
    m, e = np.frexp(x)
    return np.ldexp(np.rint(m * 256.0), e - 8)  # rint rounds halves to even


def apply_lp(lq, centroids, gamma, beta, alpha=1.0, bf16_out=True):
    """CAT Inferencing with parameters that are stored in bfloat16: the parameters are rounded with ``to_bf16``
    first, the method (``apply``) then runs on those values as it stands, and the corrected rows are rounded to
    bfloat16 at the end if ``bf16_out``.  Returns (corrected, assignments, (centroids_q, gamma_q, beta_q))."""
    cq, gq, bq = to_bf16(centroids), to_bf16(gamma), to_bf16(beta)
    out, a = apply(lq, cq, gq, bq, alpha)
    if bf16_out:
        out = to_bf16(out)
    return out, a, (cq, gq, bq)


# ---------------------------------------------------------------------------
# Lloyd iterations that leave out distance evaluations the triangle inequality makes unnecessary
# (Hamerly, "Making k-means even faster", SDM 2010).  The paper fixes no k-means variant (Sec. 4, Setup);
# this one changes the work done, never the result.
# ---------------------------------------------------------------------------
def fit_bounds(lq, fp, K, iters, seed=0, init_centroids=None):
    """``fit`` with Hamerly's bounds.  Per row i the loop keeps u(i), an upper bound on the distance to its own
    centroid, and l(i), a lower bound on the distance to every other centroid.  After an update that moves centroid
    k by p(k): u(i) += p(a(i)) and l(i) -= the largest movement among the other centroids.  With s(k) half the
    distance from centroid k to its nearest other centroid, a row with u(i) < max(s(a(i)), l(i)) is strictly nearer
    to its own centroid than to any other and is left alone; otherwise u(i) is first tightened to the true distance
    and the test repeated, and only rows that fail again have all their distances computed (nearest centroid,
    lowest index on ties, as ``assign``).  The comparisons are strict and carry a relative guard of 1e-12 against
    the rounding of the accumulated bounds, so a row is only ever left alone when its assignment cannot change.

    Returns the dict of ``fit`` without the objective trace (the distances of the rows left alone are not known),
    plus ``evaluated``: for each of the iters + 1 passes, the number of rows whose distances to all centroids were
    computed."""
    x = np.ascontiguousarray(lq, dtype=np.float32)
    xd = x.astype(np.float64)
    N, D = x.shape
    if init_centroids is None:
        cent = x[init_indices(N, K, seed)].astype(np.float64)
    else:
        cent = np.array(init_centroids, dtype=np.float64)
    guard = 1.0 + 1e-12
    a, d1, d2 = assign(x, cent, want_distances=True)
    u = np.sqrt(d1)
    l = np.sqrt(d2) if K > 1 else np.full(N, np.inf)
    evaluated = [N]
    for _ in range(iters):
        new_cent, _ = update(x, a, cent)
        p = np.sqrt(((new_cent - cent) ** 2).sum(axis=1))
        cent = new_cent
        order = np.argsort(-p, kind="stable")
        p_first = p[order[0]]
        p_second = p[order[1]] if K > 1 else 0.0
        u = u + p[a]
        l = l - np.where(a == order[0], p_second, p_first)
        if K > 1:
            cc = np.sqrt(((cent[:, None, :] - cent[None, :, :]) ** 2).sum(axis=2))
            np.fill_diagonal(cc, np.inf)
            s = 0.5 * cc.min(axis=1)
        else:
            s = np.full(1, np.inf)
        m = np.maximum(s[a], l)
        idx = np.flatnonzero(~(u * guard < m))
        if idx.size:  # tighten the upper bound to the true distance, test again
            u[idx] = np.sqrt(((xd[idx] - cent[a[idx]]) ** 2).sum(axis=1))
            idx = idx[~(u[idx] * guard < m[idx])]
        if idx.size:
            ai, e1, e2 = assign(x[idx], cent, want_distances=True)
            a[idx] = ai
            u[idx] = np.sqrt(e1)
            l[idx] = np.sqrt(e2) if K > 1 else np.inf
        evaluated.append(int(idx.size))
    gamma, beta, counts = affine(x, fp, a, K)
    return dict(centroids=cent, gamma=gamma, beta=beta, assignments=a, counts=counts,
                evaluated=np.asarray(evaluated, dtype=np.int64))
