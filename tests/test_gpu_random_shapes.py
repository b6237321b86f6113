"""Seeded random shapes through cat_fit / cat_apply against the oracle.

Shapes, dtypes, iteration counts and the kernel family are drawn from a fixed seed; the data are
small planted mixtures with a few duplicated rows (exact ties between candidates) and a few constant
channels.  The point is coverage of ragged tails, odd cluster counts and unusual D / K ratios that
the named workloads do not have.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2509_26277_amd import binding, workloads
from paper_2509_26277_amd import cat_apply, cat_fit

from parity_util import CENTROID_RTOL, RTOL, check_assignments, check_values, dev_matrix, host_matrix

pytestmark = pytest.mark.gpu


def _cases(n_cases=28, seed=20250926):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n_cases):
        dt = "bf16" if rng.random() < 0.35 else "f32"
        tile = rng.random() < 0.6
        step = (8 if dt == "bf16" else 4) if tile else (2 if dt == "bf16" else 1)
        D = int(rng.integers(1, 90)) * step
        K = int(rng.integers(1, 71))
        N = int(rng.integers(K, K + 2500))
        iters = int(rng.integers(0, 6))
        out.append((i, dt, binding.CAT_PATH_TILE if tile else binding.CAT_PATH_STREAM, N, D, K, iters))
    return out


@pytest.fixture(autouse=True)
def _auto_path_after():
    yield
    binding.select_path(binding.CAT_PATH_AUTO)


@pytest.mark.parametrize("case,dt,path,N,D,K,iters", _cases())
def test_random_shape(case, dt, path, N, D, K, iters):
    rng = np.random.default_rng(7000 + case)
    comps = max(1, min(K, 6))
    mu = 3.0 * rng.standard_normal((comps, D))
    lab = rng.integers(0, comps, N)
    fp = (mu[lab] + rng.standard_normal((N, D))).astype(np.float32)
    lq = (fp * rng.uniform(0.6, 1.4, D) + 0.3 * rng.standard_normal(D) + 0.1 * rng.standard_normal((N, D))).astype(np.float32)
    if D > 3:
        lq[:, D // 2] = 1.5  # a constant channel: variance floor in every cluster
    if N > 8:
        lq[N // 3] = lq[N // 3 + 1]  # duplicated rows
        fp[N // 3] = fp[N // 3 + 1]
    if dt == "bf16":
        lq, fp = workloads.round_to_bf16(lq), workloads.round_to_bf16(fp)
    binding.select_path(path)
    r = cat_fit(dev_matrix(lq, dt), dev_matrix(fp, dt), K, iters, seed=case)
    o = oracle.fit(lq, fp, K, iters, seed=case)
    _, d1, d2 = oracle.assign(lq, o["centroids"], want_distances=True)
    a_g = r["assignments"].cpu().numpy()
    what = f"case {case} {dt} N={N} D={D} K={K} iters={iters}"
    exempt = check_assignments(a_g, o["assignments"], d1, d2, what)
    assert r["counts"].cpu().numpy().tolist() == np.bincount(a_g, minlength=K).tolist()
    check_values(host_matrix(r["centroids"]), o["centroids"], RTOL[dt] if exempt else CENTROID_RTOL, what + " centroids")
    check_values(host_matrix(r["gamma"]), o["gamma"], RTOL[dt], what + " gamma")
    check_values(host_matrix(r["beta"]), o["beta"], RTOL[dt], what + " beta")
    alpha = 0.25 * (case % 5)
    out, a2 = cat_apply(dev_matrix(lq, dt), r["centroids"], r["gamma"], r["beta"], alpha=alpha)
    o_out, o_a = oracle.apply(lq, host_matrix(r["centroids"]), host_matrix(r["gamma"]), host_matrix(r["beta"]), alpha)
    _, e1, e2 = oracle.assign(lq, host_matrix(r["centroids"]), want_distances=True)
    ok = a2.cpu().numpy() == o_a
    assert ((e2 - e1)[~ok] <= 1e-5 * e2[~ok]).all(), what
    check_values(host_matrix(out)[ok], o_out[ok], RTOL[dt], what + " corrected")
