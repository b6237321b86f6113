"""GPU-vs-oracle parity of fits with more than 128 clusters (the paper's ablation goes up to 256), whose assignment
passes rank the clusters in two launches of 128 each when the two-part operand of all of them does not fit LDS: the
first launch hands its best score and its exact nearest centroid to the second, which ranks that pair beside its own
clusters.  The result must be the exact nearest centroid over all clusters, lowest index on ties."""
import numpy as np
import pytest
import torch

import oracle
from paper_2509_26277_amd import binding, cat_apply, cat_apply_lp, cat_assign, cat_fit, cat_params_to_bf16, workloads

from parity_util import CENTROID_RTOL, RTOL, check_assignments_lazy, check_values, dev_matrix, host_matrix

pytestmark = pytest.mark.gpu


def _mixture(seed, N, D, C, dt, spread):
    rng = np.random.default_rng(seed)
    centres = rng.standard_normal((C, D)) * spread
    lab = rng.integers(0, C, N)
    y = (centres[lab] + rng.standard_normal((N, D))).astype(np.float32)
    x = (y * rng.uniform(0.6, 1.4, D).astype(np.float32) + 0.2 * rng.standard_normal((N, D)).astype(np.float32)).astype(np.float32)
    if dt == "bf16":
        x, y = workloads.round_to_bf16(x), workloads.round_to_bf16(y)
    return x, y


@pytest.mark.parametrize("N,D,K,iters,dt,spread", [
    (6000, 260, 200, 6, "f32", 1.0),      # resident operand per launch
    (4099, 1000, 256, 5, "f32", 0.5),     # chunked operand per launch, overlapping components, ragged last tile
    (5000, 1000, 129, 5, "f32", 1.0),     # one cluster in the second launch
    (3000, 2048, 150, 4, "bf16", 1.0),    # bf16 rows
    (3000, 64, 200, 6, "f32", 1.0),       # short rows: one launch ranks all of them with the two-part operand
    (2000, 512, 192, 0, "f32", 1.0),      # no iterations
])
def test_fit_matches_the_oracle(N, D, K, iters, dt, spread):
    x, y = _mixture(N + D + K, N, D, 40, dt, spread)
    xd, yd = dev_matrix(x, dt), dev_matrix(y, dt)
    r = cat_fit(xd, yd, K, iters, seed=3)
    o = oracle.fit(x, y, K, iters, seed=3)
    a = r["assignments"].cpu().numpy()
    exempt = check_assignments_lazy(a, o["assignments"], x, o["centroids"], "assignments")
    assert r["counts"].cpu().numpy().tolist() == np.bincount(a, minlength=K).tolist()
    check_values(host_matrix(r["centroids"]), o["centroids"], CENTROID_RTOL if exempt == 0 else RTOL[dt], "centroids")
    if exempt == 0:
        check_values(host_matrix(r["gamma"]), o["gamma"], RTOL[dt], "gamma")
        check_values(host_matrix(r["beta"]), o["beta"], RTOL[dt], "beta")
    np.testing.assert_allclose(r["inertia"].cpu().numpy(), o["inertia"], rtol=1e-4)
    # inference on the fitting rows reproduces the partition
    _, a2 = cat_apply(xd, r["centroids"], r["gamma"], r["beta"])
    diff = np.flatnonzero(a2.cpu().numpy() != a)
    if diff.size:
        _, e1, e2 = oracle.assign(x[diff], host_matrix(r["centroids"]), want_distances=True)
        assert ((e2 - e1) < 1e-5 * e2).all()


def test_exact_ties_across_the_two_launches():
    # duplicated rows as seeds: clusters on either side of the split coincide; the lowest index must win, the others
    # stay empty.  Small integers: every distance is exact.
    rng = np.random.default_rng(5)
    base = rng.integers(-4, 5, (150, 264)).astype(np.float32)
    x = np.concatenate([base, base, base[:100]], axis=0)          # 400 rows, 150 distinct
    y = (2 * x + 1).astype(np.float32)
    # initial centroids: rows 0 .. 139, then their duplicates (rows 150 .. 265): cluster 140 + j coincides with cluster j
    init = np.ascontiguousarray(x[np.concatenate([np.arange(0, 140), np.arange(150, 266)])])
    xd, yd = dev_matrix(x, "f32"), dev_matrix(y, "f32")
    r = cat_fit(xd, yd, 256, 3, init_centroids=torch.from_numpy(init).cuda())
    o = oracle.fit(x, y, 256, 3, init_centroids=init.astype(np.float64))
    assert (r["assignments"].cpu().numpy() == o["assignments"]).all()
    assert (r["counts"].cpu().numpy() == o["counts"]).all()
    check_values(host_matrix(r["centroids"]), o["centroids"], CENTROID_RTOL, "centroids")


def test_logit_workload_rows_with_256_clusters():
    w = workloads.make("cfg2", n_rows=16384)
    x, y = w["lq"], w["fp"]
    xd, yd = dev_matrix(x, "f32"), dev_matrix(y, "f32")
    r = cat_fit(xd, yd, 256, 6, seed=w["seed"])
    o = oracle.fit(x, y, 256, 6, seed=w["seed"])
    a = r["assignments"].cpu().numpy()
    exempt = check_assignments_lazy(a, o["assignments"], x, o["centroids"], "assignments")
    check_values(host_matrix(r["centroids"]), o["centroids"], CENTROID_RTOL if exempt == 0 else RTOL["f32"], "centroids")
    np.testing.assert_allclose(r["inertia"].cpu().numpy(), o["inertia"], rtol=1e-4)


@pytest.mark.parametrize("N,D,K,dt", [(5000, 260, 200, "f32"), (4099, 1000, 256, "f32"), (3000, 2048, 150, "bf16"), (3000, 64, 200, "f32")])
def test_assign_and_apply_match_the_oracle(N, D, K, dt):
    """cat_assign and cat_apply with more than 128 clusters (two launches, then the map by the labels)."""
    x, _ = _mixture(N + K, N, D, 40, dt, 1.0)
    rng = np.random.default_rng(K)
    cent = x[rng.choice(N, K, replace=False)].astype(np.float32)
    cent[K - 1] = cent[3]          # an exact tie across the two halves: the lower index must win
    gamma = rng.uniform(0.7, 1.3, (K, D)).astype(np.float32)
    beta = (0.3 * rng.standard_normal((K, D))).astype(np.float32)
    xd = dev_matrix(x, dt)
    f = lambda a: torch.from_numpy(a).cuda()
    o_a, d1, d2 = oracle.assign(x, cent.astype(np.float64), want_distances=True)
    a, counts, inertia = cat_assign(xd, f(cent))
    check_assignments_lazy(a.cpu().numpy(), o_a, x, cent.astype(np.float64), "cat_assign")
    assert counts.cpu().numpy().tolist() == np.bincount(a.cpu().numpy(), minlength=K).tolist()
    np.testing.assert_allclose(float(inertia), d1.sum(), rtol=1e-4)
    assert not (a.cpu().numpy() == K - 1).any()
    for alpha in (1.0, 0.6):
        out, a2 = cat_apply(xd, f(cent), f(gamma), f(beta), alpha=alpha)
        o_out, o_a2 = oracle.apply(x, cent, gamma, beta, alpha)
        a2 = a2.cpu().numpy()
        check_assignments_lazy(a2, o_a2, x, cent.astype(np.float64), "cat_apply")
        same = a2 == o_a2
        check_values(host_matrix(out)[same], o_out[same], RTOL[dt], "corrected")
    # without the assignments output, and on the fused 16-tile kernel for comparison
    out_b, _ = cat_apply(xd, f(cent), f(gamma), f(beta), alpha=0.6, want_assignments=False)
    assert torch.equal(out_b, out)
    binding.debug_apply_kernel(1)
    try:
        out_t, a_t = cat_apply(xd, f(cent), f(gamma), f(beta), alpha=0.6)
    finally:
        binding.debug_apply_kernel(0)
    check_values(host_matrix(out_t)[a_t.cpu().numpy() == a2], host_matrix(out)[a_t.cpu().numpy() == a2], RTOL[dt], "fused kernel")
    if dt == "f32":
        cq, gq, bq = cat_params_to_bf16(f(cent)), cat_params_to_bf16(f(gamma)), cat_params_to_bf16(f(beta))
        out16, a16 = cat_apply_lp(xd, cq, gq, bq, alpha=0.6, bf16_out=True)
        o16, oa16, (ocq, _, _) = oracle.apply_lp(x, cent, gamma, beta, alpha=0.6)
        a16 = a16.cpu().numpy()
        check_assignments_lazy(a16, oa16, x, ocq, "cat_apply_lp")
        check_values(host_matrix(out16)[a16 == oa16], o16[a16 == oa16], RTOL["bf16"], "corrected, low precision")
