"""Rows or centroids with NaN / infinite entries: the result for them is unspecified, but every call returns, every label
is a cluster number, the counts add up, and the finite rows beside them get the oracle's answer."""
import numpy as np
import pytest
import torch

import oracle
from paper_2509_26277_amd import binding, cat_apply, cat_assign, cat_fit

from parity_util import RTOL, check_assignments, check_values, dev_matrix, host_matrix

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _defaults_after():
    yield
    binding.select_path(binding.CAT_PATH_AUTO)


def _rows(seed, N, D, K):
    rng = np.random.default_rng(seed)
    centres = rng.standard_normal((K, D)) * 2.0
    x = (centres[rng.integers(0, K, N)] + rng.standard_normal((N, D))).astype(np.float32)
    bad = rng.choice(N, 45, replace=False)
    x[bad[:20], rng.integers(0, D, 20)] = np.nan
    x[bad[20:30], rng.integers(0, D, 10)] = np.inf
    x[bad[30:40], rng.integers(0, D, 10)] = -np.inf
    x[bad[40:]] = np.nan
    finite = np.isfinite(x).all(axis=1)
    return x, finite


@pytest.mark.parametrize("path", [binding.CAT_PATH_AUTO, binding.CAT_PATH_TILE, binding.CAT_PATH_STREAM])
@pytest.mark.parametrize("N,D,K", [(3000, 72, 9), (2000, 257, 20)])
def test_non_finite_rows_single_passes(path, N, D, K):
    if path == binding.CAT_PATH_TILE and D % 4:
        pytest.skip("the tile kernels take rows of whole 16-byte groups")
    binding.select_path(path)
    x, finite = _rows(N + D, N, D, K)
    cent = np.ascontiguousarray(x[finite][:K])
    xd, cd = torch.from_numpy(x).cuda(), torch.from_numpy(cent).cuda()
    a, counts, _ = cat_assign(xd, cd)
    a = a.cpu().numpy()
    assert a.min() >= 0 and a.max() < K
    assert counts.cpu().numpy().tolist() == np.bincount(a, minlength=K).tolist()
    o_a, d1, d2 = oracle.assign(x[finite], cent.astype(np.float64), want_distances=True)
    check_assignments(a[finite], o_a, d1, d2, "finite rows beside non-finite ones")
    rng = np.random.default_rng(1)
    gamma = rng.uniform(0.8, 1.2, (K, D)).astype(np.float32)
    beta = rng.standard_normal((K, D)).astype(np.float32)
    out, a2 = cat_apply(xd, cd, torch.from_numpy(gamma).cuda(), torch.from_numpy(beta).cuda())
    a2 = a2.cpu().numpy()
    assert a2.min() >= 0 and a2.max() < K
    o_out, o_a2 = oracle.apply(x[finite], cent, gamma, beta)
    same = a2[finite] == o_a2
    assert same.mean() > 0.999
    check_values(host_matrix(out)[finite][same], o_out[same], RTOL["f32"], "corrected finite rows")


@pytest.mark.parametrize("path", [binding.CAT_PATH_AUTO, binding.CAT_PATH_TILE])
def test_all_centroids_non_finite(path):
    """no real score compares: a slot past the last cluster (K is not a multiple of 16) must not come out as the label"""
    binding.select_path(path)
    N, D, K = 1500, 64, 5
    x = np.random.default_rng(3).standard_normal((N, D)).astype(np.float32)
    cent = np.full((K, D), np.nan, dtype=np.float32)
    a, counts, _ = cat_assign(torch.from_numpy(x).cuda(), torch.from_numpy(cent).cuda())
    a = a.cpu().numpy()
    assert a.min() >= 0 and a.max() < K
    assert int(counts.sum().item()) == N
    out, a2 = cat_apply(torch.from_numpy(x).cuda(), torch.from_numpy(cent).cuda(),
                        torch.ones((K, D), device="cuda"), torch.zeros((K, D), device="cuda"))
    a2 = a2.cpu().numpy()
    assert a2.min() >= 0 and a2.max() < K
    np.testing.assert_array_equal(out.cpu().numpy(), x)  # gamma = 1, beta = 0 whichever cluster


@pytest.mark.parametrize("path", [binding.CAT_PATH_AUTO, binding.CAT_PATH_TILE])
def test_fit_returns_with_non_finite_rows(path):
    binding.select_path(path)
    N, D, K = 4000, 64, 6
    x, finite = _rows(9, N, D, K)
    y = np.where(np.isfinite(x), 1.5 * x + 0.1, 0.0).astype(np.float32)
    r = cat_fit(dev_matrix(x, "f32"), dev_matrix(y, "f32"), K, 4, seed=1)
    a = r["assignments"].cpu().numpy()
    assert a.min() >= 0 and a.max() < K
    assert int(r["counts"].sum().item()) == N
    assert r["counts"].cpu().numpy().tolist() == np.bincount(a, minlength=K).tolist()
