"""GPU-vs-oracle parity of the PCA front-end (Sec. 3.1; first step of Algorithms 1 and 2) and of the
pipeline built on it: fit = PCA -> project -> Lloyd on the scores -> affine fit on the full vectors;
inference = project -> nearest centroid in score space -> affine map by that label.

Eigenvectors are compared where the mathematics makes them unique: the test data have well separated
leading eigenvalues, and directions are compared through the sign convention both sides share.  Where a
group of eigenvalues is close, the span is compared instead (principal angles)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2509_26277_amd import binding, workloads
from paper_2509_26277_amd import (cat_apply_assigned, cat_assign, cat_fit, cat_pca_fit, cat_pca_project, cat_stats)

from parity_util import RTOL, check_assignments, check_values, dev_matrix, host_matrix

pytestmark = pytest.mark.gpu


def _graded(seed, N, D, dt="f32"):
    """rows with a graded spectrum (distinct leading variances) in a random orthonormal frame"""
    rng = np.random.default_rng(seed)
    scales = np.concatenate([np.linspace(6.0, 2.0, min(D, 8)), np.full(max(D - 8, 0), 0.4)])[:D]
    rot, _ = np.linalg.qr(rng.standard_normal((D, D)))
    x = ((rng.standard_normal((N, D)) * scales) @ rot + 2.0 * rng.standard_normal(D)).astype(np.float32)
    return workloads.round_to_bf16(x) if dt == "bf16" else x


@pytest.mark.parametrize("N,D,p,dt", [(700, 12, 5, "f32"), (1500, 33, 6, "f32"), (333, 7, 7, "f32"), (2000, 64, 8, "bf16"),
                                      (1000, 130, 4, "f32"), (64, 1, 1, "f32"), (50, 2, 2, "f32")])
def test_pca_fit_matches_the_oracle(N, D, p, dt):
    x = _graded(N + D, N, D, dt)
    mean_o, comps_o, evals_o = oracle.pca_fit(x, p)
    mean_g, comps_g, evals_g = cat_pca_fit(dev_matrix(x, dt), p)
    np.testing.assert_allclose(host_matrix(mean_g), mean_o, rtol=1e-6, atol=1e-6)
    np.testing.assert_allclose(evals_g.cpu().numpy(), evals_o, rtol=1e-9, atol=1e-12)
    cg = host_matrix(comps_g)
    np.testing.assert_allclose(np.linalg.norm(cg, axis=1), 1.0, atol=1e-6)
    # distinct eigenvalues (the first min(p, 8) of this spectrum): the directions themselves agree
    k = min(p, 8)
    gaps_ok = np.abs(np.diff(evals_o[:k])) > 1e-3 * evals_o[0] if k > 1 else np.array([True])
    if gaps_ok.all():
        np.testing.assert_allclose(cg[:k], comps_o[:k], atol=2e-5)
    # always: same span
    sv = np.linalg.svd(cg @ comps_o.T, compute_uv=False)
    np.testing.assert_allclose(sv, 1.0, atol=1e-5)


def test_pca_fit_with_a_repeated_eigenvalue_returns_the_same_span():
    rng = np.random.default_rng(9)
    N, D = 1200, 10
    x = rng.standard_normal((N, D)) * np.array([3, 3, 3, 1, 1, 1, 1, 1, 1, 1.0])  # three equal leading variances (in expectation)
    x = x.astype(np.float32)
    _, comps_o, evals_o = oracle.pca_fit(x, 3)
    _, comps_g, evals_g = cat_pca_fit(dev_matrix(x, "f32"), 3)
    np.testing.assert_allclose(evals_g.cpu().numpy(), evals_o, rtol=1e-9)
    sv = np.linalg.svd(host_matrix(comps_g) @ comps_o.T, compute_uv=False)
    np.testing.assert_allclose(sv, 1.0, atol=1e-5)


@pytest.mark.parametrize("N,D,p,dt", [(1000, 40, 6, "f32"), (777, 100, 70, "f32"), (1500, 64, 8, "bf16"), (5, 3, 2, "f32")])
def test_projection_matches_the_oracle(N, D, p, dt):
    x = _graded(N, N, D, dt)
    mean_g, comps_g, _ = cat_pca_fit(dev_matrix(x, dt), p)
    z_g = cat_pca_project(dev_matrix(x, dt), mean_g, comps_g)
    # teacher-forced: the oracle projects with the mean and directions the GPU holds (as floats)
    z_o = oracle.pca_project(x, host_matrix(mean_g), host_matrix(comps_g))
    check_values(host_matrix(z_g), z_o, 1e-4, "scores")


@pytest.mark.parametrize("D", [37, 1000, 264, 2048, 8])  # one channel per lane; 16-byte groups with and without a ragged last step
def test_apply_assigned_matches_the_definition(D):
    rng = np.random.default_rng(3 + D)
    N, K = 1000, 5
    for dt in ("f32", "bf16"):
        x = rng.standard_normal((N, D)).astype(np.float32)
        if dt == "bf16":
            x = workloads.round_to_bf16(x)
        g = rng.uniform(0.5, 1.5, (K, D)).astype(np.float32)
        b = rng.standard_normal((K, D)).astype(np.float32)
        a = rng.integers(0, K, N).astype(np.int32)
        a[::97] = -1  # left as they are
        for alpha in (1.0, 0.3, 0.0):
            out = cat_apply_assigned(dev_matrix(x, dt), torch.from_numpy(a).cuda(), torch.from_numpy(g).cuda(),
                                     torch.from_numpy(b).cuda(), alpha=alpha)
            xd = x.astype(np.float64)
            want = xd.copy()
            ok = a >= 0
            want[ok] = xd[ok] + alpha * ((g[a[ok]].astype(np.float64) * xd[ok] + b[a[ok]]) - xd[ok])
            check_values(host_matrix(out), want, RTOL[dt], f"apply_assigned {dt} alpha={alpha}")
            if alpha == 0.0:
                assert (host_matrix(out) == xd).all()


@pytest.mark.parametrize("name,n,p", [("cfg1", 4096, 3), ("cfg2", 1531, 15)])
def test_pipeline_with_pca_front_end(name, n, p):
    """Algorithm 1 and Algorithm 2 with pca_dim = p, step by step against the oracle."""
    w = workloads.make(name, n_rows=n)
    K, dt, iters = w["K"], w["dtype"], 5
    lq, fp = dev_matrix(w["lq"], dt), dev_matrix(w["fp"], dt)
    mean_g, comps_g, _ = cat_pca_fit(lq, p)
    z_g = cat_pca_project(lq, mean_g, comps_g)
    # the oracle clusters the scores the GPU produced (teacher-forced at the PCA boundary), so the
    # comparison of the clustering does not hinge on the last bits of the eigenvectors
    z = host_matrix(z_g).astype(np.float32)
    o = oracle.fit(z, z, K, iters, seed=w["seed"])
    r = cat_fit(z_g, z_g, K, iters, seed=w["seed"])
    _, d1, d2 = oracle.assign(z, o["centroids"], want_distances=True)
    a_g = r["assignments"].cpu().numpy()
    check_assignments(a_g, o["assignments"], d1, d2, f"{name} Lloyd on scores")
    check_values(host_matrix(r["centroids"]), o["centroids"], 1e-4, "score centroids")
    # affine fit on the full vectors by that partition
    g_g, b_g, n_g = cat_stats(lq, fp, r["assignments"], K)
    g_o, b_o, n_o = oracle.affine(w["lq"], w["fp"], a_g, K)
    assert n_g.cpu().numpy().tolist() == n_o.tolist()
    check_values(host_matrix(g_g), g_o, RTOL[dt], "gamma")
    check_values(host_matrix(b_g), b_o, RTOL[dt], "beta")
    # inference on the same rows reproduces the partition and applies the correction
    a2, _, _ = cat_assign(cat_pca_project(lq, mean_g, comps_g), r["centroids"])
    same = a2.cpu().numpy() == a_g
    _, e1, e2 = oracle.assign(z, host_matrix(r["centroids"]), want_distances=True)
    assert ((e2 - e1)[~same] <= 1e-5 * e2[~same]).all()
    out = cat_apply_assigned(lq, a2, g_g, b_g, alpha=0.6)
    xd = w["lq"].astype(np.float64)
    al = a2.cpu().numpy()
    want = xd + 0.6 * ((host_matrix(g_g)[al] * xd + host_matrix(b_g)[al]) - xd)
    check_values(host_matrix(out), want, RTOL[dt], "corrected")
    # and the whole of the PCA against the oracle's own
    mean_o, comps_o, _ = oracle.pca_fit(w["lq"], p)
    sv = np.linalg.svd(host_matrix(comps_g) @ comps_o.T, compute_uv=False)
    assert sv.min() > 1 - 1e-3, sv  # span of the leading directions (trailing ones may sit in a noise bulk)


def test_pca_argument_errors_are_statuses():
    x = torch.zeros((16, 8), device="cuda")
    with pytest.raises(binding.CatError) as e:
        cat_pca_fit(x, 9)  # p > D
    assert e.value.status == 1
    with pytest.raises(binding.CatError) as e:
        cat_pca_fit(x, 2, workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert e.value.status == 3
    with pytest.raises(binding.CatError) as e:
        cat_pca_fit(torch.zeros((4, 4096), device="cuda"), 2, workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert e.value.status == 1  # D above the limit


@pytest.mark.parametrize("name,n,p", [("cfg1", 4096, 4), ("cfg2", 1531, 12), ("cfg4", 1100, 16)])
def test_single_call_pipeline_equals_its_steps_and_the_oracle(name, n, p):
    """cat_fit_pca / cat_apply_pca against the same pipeline composed from the step calls, and the oracle
    on the boundary the steps share (the scores)."""
    from paper_2509_26277_amd import cat_apply_pca, cat_fit_pca
    w = workloads.make(name, n_rows=n)
    K, dt, iters = w["K"], w["dtype"], 4
    lq, fp = dev_matrix(w["lq"], dt), dev_matrix(w["fp"], dt)
    r = cat_fit_pca(lq, fp, K, p, iters, seed=w["seed"])
    # the steps, by hand.  (The covariance is summed with atomics, so two PCA fits agree to rounding, not bit for
    # bit; the steps after it are therefore run on the mean and directions the single call returned.)
    mean_g, comps_g, _ = cat_pca_fit(lq, p)
    torch.testing.assert_close(mean_g, r["mean"], rtol=1e-6, atol=1e-6)
    torch.testing.assert_close(comps_g, r["components"], rtol=0, atol=1e-5)
    z_g = cat_pca_project(lq, r["mean"], r["components"])
    s = cat_fit(z_g, z_g, K, iters, seed=w["seed"])
    assert torch.equal(s["assignments"], r["assignments"]) and torch.equal(s["counts"], r["counts"])
    check_values(host_matrix(r["centroids_z"]), host_matrix(s["centroids"]), 1e-6, "score centroids")
    # the oracle on the scores and on the full vectors
    z = host_matrix(z_g).astype(np.float32)
    o = oracle.fit(z, z, K, iters, seed=w["seed"])
    _, d1, d2 = oracle.assign(z, o["centroids"], want_distances=True)
    a_g = r["assignments"].cpu().numpy()
    check_assignments(a_g, o["assignments"], d1, d2, f"{name} pca pipeline")
    # the objective is a diagnostic formed as |z|^2 + (score) in float: tight clusters far from the origin of the
    # score space lose a few digits to that cancellation
    np.testing.assert_allclose(r["inertia"].cpu().numpy(), o["inertia"], rtol=1e-3)
    g_o, b_o, n_o = oracle.affine(w["lq"], w["fp"], a_g, K)
    assert r["counts"].cpu().numpy().tolist() == n_o.tolist()
    check_values(host_matrix(r["gamma"]), g_o, RTOL[dt], "gamma")
    check_values(host_matrix(r["beta"]), b_o, RTOL[dt], "beta")
    # inference
    for alpha in (1.0, 0.4):
        out, a2 = cat_apply_pca(lq, r["mean"], r["components"], r["centroids_z"], r["gamma"], r["beta"], alpha=alpha)
        al = a2.cpu().numpy()
        same = al == a_g
        _, e1, e2 = oracle.assign(z, host_matrix(r["centroids_z"]), want_distances=True)
        assert ((e2 - e1)[~same] <= 1e-5 * e2[~same]).all()
        xd = w["lq"].astype(np.float64)
        want = xd + alpha * ((host_matrix(r["gamma"])[al] * xd + host_matrix(r["beta"])[al]) - xd)
        check_values(host_matrix(out), want, RTOL[dt], f"corrected alpha={alpha}")
    out2, none = cat_apply_pca(lq, r["mean"], r["components"], r["centroids_z"], r["gamma"], r["beta"], want_assignments=False)
    assert none is None and torch.equal(out2, cat_apply_pca(lq, r["mean"], r["components"], r["centroids_z"], r["gamma"], r["beta"])[0])


@pytest.mark.parametrize("name,n,p", [("cfg2", 2000, 50), ("cfg2", 777, 20), ("cfg4", 1500, 7), ("cfg1", 4096, 64)])
def test_fused_inference_equals_the_step_sequence(name, n, p):
    """cat_apply_pca runs as one kernel where the shape allows it; with the streaming path selected it runs
    projection, assignment in score space and the labelled affine map one after the other.  Same scores (the same
    MFMA sequence), the same exact nearest centroid, the same fp32 affine map: identical outputs."""
    from paper_2509_26277_amd import cat_apply_pca, cat_fit_pca
    w = workloads.make(name, n_rows=n)
    K, dt = w["K"], w["dtype"]
    lq, fp = dev_matrix(w["lq"], dt), dev_matrix(w["fp"], dt)
    r = cat_fit_pca(lq, fp, K, p, 3, seed=w["seed"])
    args = (lq, r["mean"], r["components"], r["centroids_z"], r["gamma"], r["beta"])
    try:
        fused, a_fused = cat_apply_pca(*args, alpha=0.7)
        binding.select_path(binding.CAT_PATH_STREAM)
        steps, a_steps = cat_apply_pca(*args, alpha=0.7)
    finally:
        binding.select_path(binding.CAT_PATH_AUTO)
    assert torch.equal(a_fused, a_steps)
    assert torch.equal(fused, steps)
    # and the assignments are those of the fit on the same rows
    assert torch.equal(a_fused, r["assignments"])
