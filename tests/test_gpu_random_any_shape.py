"""Seeded random shapes with NO constraint on the row length, through the default path selection: whatever kernels the
library picks (tile kernels, a zero-padded copy for the Lloyd loop, the word-by-word inference instances, the LDS
streaming kernel), fit, inference and assignment must match the oracle to the usual bars, and the calls must agree with
each other."""
import numpy as np
import pytest
import torch

import oracle
from paper_2509_26277_amd import cat_apply, cat_assign, cat_fit, cat_fit_multi_k, workloads

from parity_util import CENTROID_RTOL, RTOL, check_assignments_lazy, check_values, dev_matrix, host_matrix

pytestmark = pytest.mark.gpu


def _cases(n_cases=24, seed=20251201):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n_cases):
        dt = "bf16" if rng.random() < 0.3 else "f32"
        D = int(rng.integers(1, 1100 if i % 3 == 0 else 300))
        if dt == "bf16":
            D = 2 * max(1, D // 2)
        K = int(rng.choice([1, 2, 3, 7, 16, 33, 64, 100, 130, 200]))
        N = int(rng.integers(max(K, 2), K + 1500))
        iters = int(rng.integers(0, 6))
        out.append((i, dt, N, D, K, iters, bool(rng.random() < 0.5)))
    return out


@pytest.mark.parametrize("case,dt,N,D,K,iters,bounds", _cases())
def test_random_shape(case, dt, N, D, K, iters, bounds):
    rng = np.random.default_rng(7000 + case)
    C = max(2, min(K, 6))
    mu = rng.standard_normal((C, D)) * 2
    y = (mu[rng.integers(0, C, N)] + rng.standard_normal((N, D))).astype(np.float32)
    x = (y * rng.uniform(0.7, 1.3, D).astype(np.float32) + 0.1 * rng.standard_normal((N, D)).astype(np.float32)).astype(np.float32)
    if dt == "bf16":
        x, y = workloads.round_to_bf16(x), workloads.round_to_bf16(y)
    xd, yd = dev_matrix(x, dt), dev_matrix(y, dt)
    r = cat_fit(xd, yd, K, iters, seed=case, bounds=bounds, early_stop=not bounds and case % 3 == 0)
    o = oracle.fit(x, y, K, iters, seed=case)
    exempt = check_assignments_lazy(r["assignments"].cpu().numpy(), o["assignments"], x, o["centroids"], "fit")
    if exempt == 0:
        assert (r["counts"].cpu().numpy() == o["counts"]).all()
        check_values(host_matrix(r["centroids"]), o["centroids"], CENTROID_RTOL, "centroids")
        check_values(host_matrix(r["gamma"]), o["gamma"], RTOL[dt], "gamma")
        check_values(host_matrix(r["beta"]), o["beta"], RTOL[dt], "beta")
    # inference and assignment with the fitted parameters
    cent, gamma, beta = (host_matrix(r[k]) for k in ("centroids", "gamma", "beta"))
    out, a = cat_apply(xd, r["centroids"], r["gamma"], r["beta"], alpha=0.7)
    o_out, o_a = oracle.apply(x, cent, gamma, beta, 0.7)
    a = a.cpu().numpy()
    check_assignments_lazy(a, o_a, x, cent, "inference")
    check_values(host_matrix(out)[a == o_a], o_out[a == o_a], RTOL[dt], "corrected")
    a2, counts2, inertia2 = cat_assign(xd, r["centroids"])
    a2 = a2.cpu().numpy()
    check_assignments_lazy(a2, o_a, x, cent, "assignment")
    assert counts2.cpu().numpy().tolist() == np.bincount(a2, minlength=K).tolist()
    _, d1, _ = oracle.assign(x, cent, want_distances=True)
    assert float(inertia2) == pytest.approx(d1.sum(), rel=1e-4, abs=1e-6 * float((x.astype(np.float64) ** 2).sum()))
    # the same count inside a list of two equals the single fit
    if iters >= 1 and K <= 64:
        m = cat_fit_multi_k(xd, yd, [max(1, K // 2), K], iters, seed=case)
        s = cat_fit(xd, yd, K, iters, seed=case)
        assert torch.equal(m[1]["assignments"], s["assignments"]) and torch.equal(m[1]["centroids"], s["centroids"])
