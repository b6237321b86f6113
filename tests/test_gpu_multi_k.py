"""GPU-vs-oracle parity of the fits for a grid of cluster counts (cat_fit_multi_k).

The oracle is a plain loop over its pinned ``fit`` (``oracle.fit_multi_k``).  The library runs the Lloyd loops of
several cluster counts side by side where the shape allows it; every entry must equal the oracle's fit of that count
to the usual tolerances, and the library's own single ``cat_fit`` of that count: centroids, assignments and counts bit
for bit, gamma and beta to rounding (sharing the reads changes nothing that is computed)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2509_26277_amd import cat_fit, cat_fit_multi_k, workloads
from paper_2509_26277_amd.binding import CatError, debug_multi_group_tiles

from parity_util import CENTROID_RTOL, RTOL, check_assignments_lazy, check_values, dev_matrix, host_matrix

pytestmark = pytest.mark.gpu

PAPER_GRID = [1, 8, 16, 24, 32, 48, 64, 96, 128, 192, 256]  # the cluster counts of the paper's ablation figures


@pytest.fixture(autouse=True)
def _default_groups_after():
    yield
    debug_multi_group_tiles(0)


def _mixture(seed, N, D, C, dt):
    rng = np.random.default_rng(seed)
    centres = rng.standard_normal((C, D)) * 2.0
    lab = rng.integers(0, C, N)
    y = (centres[lab] + rng.standard_normal((N, D))).astype(np.float32)
    x = (y * rng.uniform(0.6, 1.4, D).astype(np.float32) + 0.2 * rng.standard_normal((N, D)).astype(np.float32)).astype(np.float32)
    if dt == "bf16":
        x, y = workloads.round_to_bf16(x), workloads.round_to_bf16(y)
    return x, y


def _same_as_single(r, s):
    for key in ("centroids", "assignments", "counts"):
        assert torch.equal(r[key], s[key]), key
    for key in ("gamma", "beta"):  # (the statistics are summed with atomics: two runs agree to the last bits, not bit for bit)
        torch.testing.assert_close(r[key], s[key], rtol=1e-5, atol=1e-6)
    # The objective is a diagnostic summed from the kernel's scores, and the two calls may run different variants of
    # the kernel: a group always ranks with the two-part operand, a single fit whose operand then fits LDS whole may
    # rank with one part (scores good to 2^-8 of |x||c|; the decision itself is re-ranked exactly either way).
    np.testing.assert_allclose(r["inertia"].cpu().numpy(), s["inertia"].cpu().numpy(), rtol=5e-4)


def _same_as_oracle(r, o, x, dt, what):
    a = r["assignments"].cpu().numpy()
    # trajectories are compared as they are: a flipped near-tie would show as a clear difference later on
    assert (a == o["assignments"]).all(), what
    assert (r["counts"].cpu().numpy() == o["counts"]).all(), what
    check_values(host_matrix(r["centroids"]), o["centroids"], CENTROID_RTOL, what + " centroids")
    check_values(host_matrix(r["gamma"]), o["gamma"], RTOL[dt], what + " gamma")
    check_values(host_matrix(r["beta"]), o["beta"], RTOL[dt], what + " beta")
    np.testing.assert_allclose(r["inertia"].cpu().numpy(), o["inertia"], rtol=1e-4)


@pytest.mark.parametrize("N,D,Ks,iters,dt", [
    (3000, 64, [1, 5, 16, 17], 6, "f32"),                 # one group of five tiles
    (2500, 136, [9, 3, 40], 5, "bf16"),                   # a ragged last chunk of channels, bf16 rows
    (4099, 260, [2, 33, 7, 100, 64], 5, "f32"),           # rows not a multiple of 16; three groups
    (1500, 37, [4, 6], 3, "f32"),                         # D not a multiple of 4: a group on a zero-padded copy of the rows
    (2000, 32, [300, 8, 12], 4, "f32"),                   # an entry the tile kernels cannot take, then a group
    (1200, 48, [7], 4, "f32"),                            # a list of one
    (900, 16, [3, 5], 0, "f32"),                          # no iterations
    (2048, 64, [4, 4, 4], 7, "f32"),                      # the same count three times
])
def test_every_entry_matches_the_oracle_and_the_single_fit(N, D, Ks, iters, dt):
    x, y = _mixture(N + D, N, D, 6, dt)
    xd, yd = dev_matrix(x, dt), dev_matrix(y, dt)
    res = cat_fit_multi_k(xd, yd, Ks, iters, seed=11)
    ora = oracle.fit_multi_k(x, y, Ks, iters, seed=11)
    assert len(res) == len(Ks)
    for K, r, o in zip(Ks, res, ora):
        _same_as_single(r, cat_fit(xd, yd, K, iters, seed=11))
        _same_as_oracle(r, o, x, dt, f"K={K}")


def test_paper_grid_small_rows():
    N, D, iters = 8192, 64, 6
    x, y = _mixture(77, N, D, 24, "f32")
    xd, yd = dev_matrix(x, "f32"), dev_matrix(y, "f32")
    res = cat_fit_multi_k(xd, yd, PAPER_GRID, iters, seed=3)
    ora = oracle.fit_multi_k(x, y, PAPER_GRID, iters, seed=3)
    for K, r, o in zip(PAPER_GRID, res, ora):
        _same_as_oracle(r, o, x, "f32", f"K={K}")


@pytest.mark.parametrize("tiles", [1, 2, 8])
def test_results_do_not_depend_on_the_grouping(tiles):
    N, D, Ks, iters = 3000, 128, [3, 20, 16, 50, 9, 64], 6
    x, y = _mixture(5, N, D, 8, "f32")
    xd, yd = dev_matrix(x, "f32"), dev_matrix(y, "f32")
    ref = cat_fit_multi_k(xd, yd, Ks, iters, seed=2)
    debug_multi_group_tiles(tiles)
    got = cat_fit_multi_k(xd, yd, Ks, iters, seed=2)
    for r, g in zip(ref, got):
        _same_as_single(g, r)


def test_empty_clusters_and_duplicate_rows_inside_a_group():
    # many identical rows: seeded centroids coincide, the later duplicates stay empty (lowest index wins the tie)
    rng = np.random.default_rng(8)
    base = rng.standard_normal((5, 32)).astype(np.float32)
    x = np.repeat(base, 400, axis=0)
    y = (x * 1.5 + 0.25).astype(np.float32)
    xd, yd = dev_matrix(x, "f32"), dev_matrix(y, "f32")
    Ks = [8, 3, 20]
    res = cat_fit_multi_k(xd, yd, Ks, 4, seed=1)
    ora = oracle.fit_multi_k(x, y, Ks, 4, seed=1)
    for K, r, o in zip(Ks, res, ora):
        assert (r["assignments"].cpu().numpy() == o["assignments"]).all()
        assert (r["counts"].cpu().numpy() == o["counts"]).all()
        check_values(host_matrix(r["centroids"]), o["centroids"], CENTROID_RTOL, "centroids")
        check_values(host_matrix(r["gamma"]), o["gamma"], 1e-4, "gamma")
        check_values(host_matrix(r["beta"]), o["beta"], 1e-4, "beta")


def test_paper_grid_on_all_rows_of_the_logit_workload():
    w = workloads.make("cfg2")
    x, y = w["lq"], w["fp"]
    xd, yd = dev_matrix(x, "f32"), dev_matrix(y, "f32")
    iters = 5
    res = cat_fit_multi_k(xd, yd, PAPER_GRID, iters, seed=w["seed"])
    for K, r in zip(PAPER_GRID, res):
        _same_as_single(r, cat_fit(xd, yd, K, iters, seed=w["seed"]))
    for K in (8, 24):  # the whole oracle fit for two members of the grid
        r = res[PAPER_GRID.index(K)]
        o = oracle.fit(x, y, K, iters, seed=w["seed"])
        n_exempt = check_assignments_lazy(r["assignments"].cpu().numpy(), o["assignments"], x, o["centroids"], f"K={K}")
        if n_exempt == 0:
            _same_as_oracle(r, o, x, "f32", f"K={K}")


def test_bad_arguments_are_refused():
    x = torch.zeros((64, 8), device="cuda")
    for Ks in ([], [0], [65], [2] * 65):
        with pytest.raises(CatError):
            cat_fit_multi_k(x, x, Ks, 1)
