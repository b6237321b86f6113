"""The LDS streaming kernel (shapes outside the matrix-core kernels: rows that are not whole 16-byte groups,
more than 256 clusters) against the oracle, through the default path selection.

Every shape here is refused by the tile kernels, so CAT_PATH_AUTO runs k_assign_lds for the assignment passes
of cat_fit / cat_assign and for cat_apply.  Bars as everywhere: assignments identical except rows whose oracle
top-2 gap is below 1e-5 relative, values within 1e-4 (fp32 rows) / 2e-2 (bf16 rows), centroids at 1e-6.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2509_26277_amd import binding, workloads
from paper_2509_26277_amd import cat_apply, cat_assign, cat_fit

from parity_util import CENTROID_RTOL, RTOL, check_assignments, check_values, dev_matrix, f32_round, host_matrix

pytestmark = pytest.mark.gpu

# (N, D, K, dtype): one cluster group of 16 / 32 / 64, several groups (K > 64), K > 256, a ragged last tile of
# the 256-row tiles, a single short tile, rows of a few channels
SHAPES = [
    (3000, 1001, 16, "f32"), (777, 7, 5, "f32"), (2500, 129, 33, "f32"), (1500, 61, 70, "f32"),
    (1200, 50, 300, "f32"), (2000, 64, 300, "f32"), (256, 3, 2, "f32"), (100, 1, 3, "f32"),
    (2100, 1002, 16, "bf16"), (900, 30, 40, "bf16"), (700, 2, 130, "bf16"),
]


def _data(N, D, K, dt, seed):
    rng = np.random.default_rng(seed)
    comps = max(1, min(K, 7))
    mu = 3.0 * rng.standard_normal((comps, D))
    lab = rng.integers(0, comps, N)
    fp = (mu[lab] + rng.standard_normal((N, D))).astype(np.float32)
    lq = (fp * rng.uniform(0.6, 1.4, D) + 0.3 * rng.standard_normal(D) + 0.1 * rng.standard_normal((N, D))).astype(np.float32)
    if D > 3:
        lq[:, D // 2] = 1.5
    if N > 8:
        lq[N // 3] = lq[N // 3 + 1]
        fp[N // 3] = fp[N // 3 + 1]
    if dt == "bf16":
        lq, fp = workloads.round_to_bf16(lq), workloads.round_to_bf16(fp)
    return lq, fp


@pytest.fixture(autouse=True)
def _auto_path():
    binding.select_path(binding.CAT_PATH_AUTO)
    binding.debug_padded_fit(False)  # the Lloyd loops here are this kernel's, not those on a zero-padded copy of the rows
    binding.debug_apply_kernel(1)    # and the inference passes too, not the row-tile kernel's word-by-word instances
    yield
    binding.select_path(binding.CAT_PATH_AUTO)
    binding.debug_padded_fit(True)
    binding.debug_apply_kernel(0)


@pytest.mark.parametrize("N,D,K,dt", SHAPES)
def test_shapes_are_outside_the_tile_kernels(N, D, K, dt):
    binding.select_path(binding.CAT_PATH_TILE)
    lq, _ = _data(N, D, K, dt, 1)
    cent = torch.from_numpy(np.ascontiguousarray(lq[:K], dtype=np.float32)).cuda()
    with pytest.raises(binding.CatError):
        cat_assign(dev_matrix(lq, dt), cent)


@pytest.mark.parametrize("N,D,K,dt", SHAPES)
def test_assign_step(N, D, K, dt):
    lq, fp = _data(N, D, K, dt, 100 + N)
    o = oracle.fit(lq, fp, K, iters=2, seed=5)
    cent = f32_round(o["centroids"])
    a_o, d1, d2 = oracle.assign(lq, cent, want_distances=True)
    a_g, counts, inertia = cat_assign(dev_matrix(lq, dt), torch.from_numpy(cent.astype(np.float32)).cuda())
    a_g = a_g.cpu().numpy()
    check_assignments(a_g, a_o, d1, d2, f"assign {N}x{D} K={K} {dt}")
    assert counts.cpu().numpy().tolist() == np.bincount(a_g, minlength=K).tolist()
    assert inertia.item() == pytest.approx(d1.sum(), rel=1e-4)


@pytest.mark.parametrize("K,D", [(6, 5), (70, 9), (300, 6)])
def test_exact_ties_go_to_the_lowest_index(K, D):
    # duplicated centroids (every row is exactly tied between a centroid and its copies) and rows at the exact
    # midpoint of two centroids with power-of-two coordinates: no exemption, bit for bit
    rng = np.random.default_rng(K)
    base = rng.integers(-4, 5, size=(K, D)).astype(np.float32) * 0.5
    base[K // 2] = base[1]
    base[K - 1] = base[0]
    lab = rng.integers(0, K, 1500)
    lq = (base[lab] + rng.integers(-1, 2, size=(1500, D)) * 0.125).astype(np.float32)
    lq[:50] = 0.5 * (base[2] + base[3])  # midpoints
    a_o, d1, d2 = oracle.assign(lq, base.astype(np.float64), want_distances=True)
    a_g, _, _ = cat_assign(dev_matrix(lq, "f32"), torch.from_numpy(base).cuda())
    assert (a_g.cpu().numpy() == a_o).all()
    assert (d1 == d2).any()


@pytest.mark.parametrize("N,D,K,dt", SHAPES)
def test_fit_and_apply(N, D, K, dt):
    lq, fp = _data(N, D, K, dt, 300 + D)
    iters = 3
    r = cat_fit(dev_matrix(lq, dt), dev_matrix(fp, dt), K, iters, seed=11)
    o = oracle.fit(lq, fp, K, iters, seed=11)
    _, d1, d2 = oracle.assign(lq, o["centroids"], want_distances=True)
    what = f"fit {N}x{D} K={K} {dt}"
    a_g = r["assignments"].cpu().numpy()
    exempt = check_assignments(a_g, o["assignments"], d1, d2, what)
    assert r["counts"].cpu().numpy().tolist() == np.bincount(a_g, minlength=K).tolist()
    check_values(host_matrix(r["centroids"]), o["centroids"], RTOL[dt] if exempt else CENTROID_RTOL, what + " centroids")
    check_values(host_matrix(r["gamma"]), o["gamma"], RTOL[dt], what + " gamma")
    check_values(host_matrix(r["beta"]), o["beta"], RTOL[dt], what + " beta")
    for alpha in (1.0, 0.25):
        out, a2 = cat_apply(dev_matrix(lq, dt), r["centroids"], r["gamma"], r["beta"], alpha=alpha)
        o_out, o_a = oracle.apply(lq, host_matrix(r["centroids"]), host_matrix(r["gamma"]), host_matrix(r["beta"]), alpha)
        _, e1, e2 = oracle.assign(lq, host_matrix(r["centroids"]), want_distances=True)
        n_bad = check_assignments(a2.cpu().numpy(), o_a, e1, e2, what + " apply")
        ok = a2.cpu().numpy() == o_a
        assert n_bad == (~ok).sum()
        check_values(host_matrix(out)[ok], o_out[ok], RTOL[dt], what + " corrected")


def test_same_result_as_the_direct_form_kernel():
    # the two streaming families (fp32 scores + exact re-rank, and direct-form double throughout) agree bit for bit
    N, D, K = 5000, 203, 37
    lq, fp = _data(N, D, K, "f32", 9)
    cent = torch.from_numpy(np.ascontiguousarray(lq[:K])).cuda()
    a1, c1, _ = cat_assign(dev_matrix(lq, "f32"), cent)
    binding.select_path(binding.CAT_PATH_STREAM)
    a2, c2, _ = cat_assign(dev_matrix(lq, "f32"), cent)
    assert torch.equal(a1, a2) and torch.equal(c1, c2)
