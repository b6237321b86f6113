"""Pins of the PCA part of the oracle (Sec. 3.1; first step of Algorithms 1 and 2) against what the
mathematics and independent library routines fix: the SVD of the centred data, scikit-learn's PCA,
orthonormality and decorrelation, a planted subspace, and the fact that a full-rank PCA is a rigid
motion (which is why clustering raw LQ vectors is the pca_dim = D case of the paper's pipeline)."""
import numpy as np
import pytest

import oracle


def _data(seed, N=500, D=12):
    rng = np.random.default_rng(seed)
    scales = np.linspace(4.0, 0.3, D)  # distinct variances: distinct eigenvalues
    rot, _ = np.linalg.qr(rng.standard_normal((D, D)))
    return ((rng.standard_normal((N, D)) * scales) @ rot + rng.standard_normal(D) * 3).astype(np.float32)


def _fix_sign(v):
    v = v.copy()
    for c in range(v.shape[0]):
        j = int(np.argmax(np.abs(v[c])))
        if v[c, j] < 0:
            v[c] = -v[c]
    return v


def test_covariance_is_numpy_cov_with_population_divisor():
    x = _data(1)
    mean, cov = oracle.covariance(x)
    np.testing.assert_allclose(mean, x.astype(np.float64).mean(axis=0), rtol=1e-13)
    np.testing.assert_allclose(cov, np.cov(x.astype(np.float64), rowvar=False, bias=True), rtol=1e-11, atol=1e-13)
    assert (cov == cov.T).all()


def test_directions_are_right_singular_vectors_of_the_centred_data():
    x = _data(2)
    p = 5
    mean, comps, evals = oracle.pca_fit(x, p)
    xc = x.astype(np.float64) - x.astype(np.float64).mean(axis=0)
    _, s, vt = np.linalg.svd(xc, full_matrices=False)
    np.testing.assert_allclose(evals, s[:p] ** 2 / x.shape[0], rtol=1e-10)
    np.testing.assert_allclose(comps, _fix_sign(vt[:p]), atol=1e-9)
    assert (np.diff(evals) <= 0).all()
    for c in range(p):
        assert comps[c, np.argmax(np.abs(comps[c]))] > 0


def test_against_scikit_learn():
    decomposition = pytest.importorskip("sklearn.decomposition")
    x = _data(3, N=400, D=9)
    p = 4
    mean, comps, evals = oracle.pca_fit(x, p)
    sk = decomposition.PCA(n_components=p, svd_solver="full").fit(x.astype(np.float64))
    np.testing.assert_allclose(mean, sk.mean_, rtol=1e-12)
    np.testing.assert_allclose(comps, _fix_sign(sk.components_), atol=1e-9)
    # scikit-learn divides by N - 1
    np.testing.assert_allclose(evals, sk.explained_variance_ * (x.shape[0] - 1) / x.shape[0], rtol=1e-10)
    z = oracle.pca_project(x, mean, comps)
    zs = sk.transform(x.astype(np.float64)) * np.sign((comps * sk.components_).sum(axis=1))
    np.testing.assert_allclose(z, zs, atol=1e-9)


def test_orthonormal_directions_and_decorrelated_scores():
    x = _data(4)
    p = 6
    mean, comps, evals = oracle.pca_fit(x, p)
    np.testing.assert_allclose(comps @ comps.T, np.eye(p), atol=1e-12)
    z = oracle.pca_project(x, mean, comps)
    np.testing.assert_allclose(z.mean(axis=0), 0, atol=1e-9)
    np.testing.assert_allclose(z.T @ z / x.shape[0], np.diag(evals), atol=1e-9)
    _, cov = oracle.covariance(x)
    np.testing.assert_allclose(cov @ comps.T, comps.T * evals, atol=1e-9)  # eigen equation


def test_planted_subspace_is_recovered():
    rng = np.random.default_rng(5)
    D, r, N = 20, 3, 800
    basis, _ = np.linalg.qr(rng.standard_normal((D, r)))
    x = ((rng.standard_normal((N, r)) * [5.0, 3.0, 2.0]) @ basis.T + 1e-3 * rng.standard_normal((N, D))).astype(np.float32)
    _, comps, evals = oracle.pca_fit(x, r)
    # principal angles between the spans
    sv = np.linalg.svd(comps @ basis, compute_uv=False)
    np.testing.assert_allclose(sv, 1.0, atol=1e-6)
    assert evals[-1] > 1.0


def test_full_rank_pca_is_a_rigid_motion_so_kmeans_does_not_see_it():
    x = _data(6, N=300, D=7)
    mean, comps, _ = oracle.pca_fit(x, x.shape[1])
    z = oracle.pca_project(x, mean, comps)
    xd = x.astype(np.float64)
    d_x = ((xd[:40, None, :] - xd[None, 40:80, :]) ** 2).sum(-1)
    d_z = ((z[:40, None, :] - z[None, 40:80, :]) ** 2).sum(-1)
    np.testing.assert_allclose(d_z, d_x, rtol=1e-10)
    np.testing.assert_allclose(z @ comps + mean, xd, atol=1e-9)  # and it inverts exactly
    # same partition from Lloyd in either space (centroids mapped by the same motion)
    init = xd[[3, 77, 150]]
    a_x = oracle.fit(x, x, 3, 5, init_centroids=init)["assignments"]
    zf = z.astype(np.float32)
    init_z = (init - mean) @ comps.T
    a_z = oracle.fit(zf, zf, 3, 5, init_centroids=init_z)["assignments"]
    assert (a_x != a_z).mean() < 0.01  # z is rounded to float for the second run: allow near-ties to flip


def test_projection_definition_on_a_hand_case():
    x = np.array([[1, 0], [3, 0], [1, 2], [3, 2]], dtype=np.float32)  # variance 1 along each axis
    mean = np.array([2.0, 1.0])
    comps = np.array([[0.6, 0.8]])
    z = oracle.pca_project(x, mean, comps)
    np.testing.assert_allclose(z[:, 0], [-1.4, -0.2, 0.2, 1.4], rtol=1e-15)
