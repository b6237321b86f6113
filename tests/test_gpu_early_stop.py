"""GPU-vs-oracle parity of cat_fit_early_stop: the Lloyd loop that leaves out the passes after the partition has
stopped changing.  Every output is held to the bar of cat_fit (assignments exact up to rows the oracle itself calls
tied, values within the relative tolerance of the dtype); the number of passes left out is an integer fixed by the
index of the first repeated partition, which the oracle reports, and is compared exactly."""
import numpy as np
import pytest
import torch

import oracle
from paper_2509_26277_amd import binding, cat_fit, workloads

from parity_util import RTOL, check_assignments, check_values, dev_matrix, host_matrix

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _auto_path():
    binding.select_path(binding.CAT_PATH_AUTO)
    yield
    binding.select_path(binding.CAT_PATH_AUTO)


def _mixture(seed, N, D, K, spread, dt):
    rng = np.random.default_rng(seed)
    centres = rng.standard_normal((K, D)) * spread
    x = (centres[rng.integers(0, K, N)] + rng.standard_normal((N, D))).astype(np.float32)
    y = (1.1 * x + 0.05 * rng.standard_normal((N, D))).astype(np.float32)
    if dt == "bf16":
        x, y = workloads.round_to_bf16(x), workloads.round_to_bf16(y)
    return x, y


def _expected_skips(stable_at, iters):
    return 0 if stable_at < 0 else max(0, iters - 1 - max(stable_at, 2))


CASES = [
    # seed, N, D, K, spread, dtype, iters
    (0, 4096, 64, 4, 3.0, "f32", 30),     # settles after a few passes: most of the loop is left out
    (1, 6007, 256, 8, 1.5, "f32", 25),    # ragged last tile
    (2, 3000, 128, 6, 2.0, "bf16", 20),
    (3, 5000, 32, 16, 0.3, "f32", 6),     # overlapping clusters, few passes: never settles, nothing left out
    (4, 2048, 1000, 16, 1.0, "f32", 30),  # the logit shape
    (5, 1500, 64, 3, 4.0, "f32", 3),      # too short for a pass to be left out
    (6, 1500, 64, 3, 4.0, "f32", 4),      # exactly one candidate pass
    (7, 999, 64, 1, 1.0, "f32", 9),       # one cluster: pass 1 already repeats pass 0
]


@pytest.mark.parametrize("seed,N,D,K,spread,dt,iters", CASES)
def test_outputs_and_skipped_passes_match_the_oracle(seed, N, D, K, spread, dt, iters):
    x, y = _mixture(seed, N, D, K, spread, dt)
    o = oracle.fit_early_stop(x, y, K, iters, seed=seed)
    r = cat_fit(dev_matrix(x, dt), dev_matrix(y, dt), K, iters, seed=seed, early_stop=True)
    _, d1, d2 = oracle.assign(x, o["centroids"], want_distances=True)
    a_g = r["assignments"].cpu().numpy()
    moved = check_assignments(a_g, o["assignments"], d1, d2, "early stop")
    assert r["counts"].cpu().numpy().tolist() == np.bincount(a_g, minlength=K).tolist()
    check_values(host_matrix(r["centroids"]), o["centroids"], RTOL[dt], "centroids")
    check_values(host_matrix(r["gamma"]), o["gamma"], RTOL[dt], "gamma")
    check_values(host_matrix(r["beta"]), o["beta"], RTOL[dt], "beta")
    np.testing.assert_allclose(r["inertia"].cpu().numpy(), o["inertia"], rtol=1e-4)
    if moved == 0:  # the two sides saw the same partitions: the same passes repeat
        assert int(r["passes_skipped"].item()) == _expected_skips(int(o["stable_at"]), iters), o["stable_at"]
    assert 0 <= int(r["passes_skipped"].item()) <= max(0, iters - 3)


def test_empty_clusters_and_duplicate_rows():
    """rows drawn from three distinct vectors, K = 5: duplicate initial centroids leave clusters empty (they keep
    their centroid, gamma = 1, beta = 0), the partition repeats at once"""
    rng = np.random.default_rng(12)
    base = rng.standard_normal((3, 64)).astype(np.float32)
    x = base[rng.integers(0, 3, 2000)]
    y = (0.9 * x + 0.1).astype(np.float32)
    o = oracle.fit_early_stop(x, y, 5, 12, seed=4)
    assert (o["counts"] == 0).any() and 1 <= o["stable_at"] <= 2
    r = cat_fit(dev_matrix(x, "f32"), dev_matrix(y, "f32"), 5, 12, seed=4, early_stop=True)
    assert (r["assignments"].cpu().numpy() == o["assignments"]).all()
    assert r["counts"].cpu().numpy().tolist() == o["counts"].tolist()
    assert int(r["passes_skipped"].item()) == _expected_skips(int(o["stable_at"]), 12) == 9
    check_values(host_matrix(r["centroids"]), o["centroids"], RTOL["f32"], "centroids")
    empty = o["counts"] == 0
    assert (host_matrix(r["gamma"])[empty] == 1.0).all() and (host_matrix(r["beta"])[empty] == 0.0).all()
    # every row coincides with its centroid: the objective is zero up to the rounding of the fp32 scores
    np.testing.assert_allclose(r["inertia"].cpu().numpy(), o["inertia"], rtol=1e-4, atol=1e-5 * float((x.astype(np.float64) ** 2).sum()))


def test_full_logit_workload_never_settles_and_matches_the_full_fit():
    """all of cfg2 (65,536 x 1000, K = 16, 30 iterations): no pass repeats its predecessor, nothing is left out"""
    w = workloads.make("cfg2")
    o = oracle.fit_early_stop(w["lq"], w["fp"], w["K"], w["iters"], seed=w["seed"])
    assert o["stable_at"] == -1
    r = cat_fit(dev_matrix(w["lq"], "f32"), dev_matrix(w["fp"], "f32"), w["K"], w["iters"], seed=w["seed"], early_stop=True)
    assert int(r["passes_skipped"].item()) == 0
    _, d1, d2 = oracle.assign(w["lq"], o["centroids"], want_distances=True)
    check_assignments(r["assignments"].cpu().numpy(), o["assignments"], d1, d2, "cfg2 early stop")
    check_values(host_matrix(r["centroids"]), o["centroids"], RTOL["f32"], "centroids")
    np.testing.assert_allclose(r["inertia"].cpu().numpy(), o["inertia"], rtol=1e-4)


def test_the_cases_cover_both_outcomes():
    """guards the case table: at least one case stops early by a wide margin, one never settles (CPU only)"""
    stops = []
    for seed, N, D, K, spread, dt, iters in CASES:
        x, y = _mixture(seed, N, D, K, spread, dt)
        stops.append(_expected_skips(int(oracle.fit_early_stop(x, y, K, iters, seed=seed)["stable_at"]), iters))
    assert max(stops) >= 10 and min(stops) == 0 and stops[3] == 0 and stops[6] == 1


@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_same_outputs_as_the_full_loop(dt):
    """against cat_fit itself, as a property at a size the oracle is not run at: the integer outputs and the
    centroids bit for bit (both loops end with the same preparation from the same sums), the rest to rounding"""
    x, y = _mixture(21, 60000, 256, 4, 3.0, dt)
    xd, yd = dev_matrix(x, dt), dev_matrix(y, dt)
    full = cat_fit(xd, yd, 4, 40, seed=5)
    r = cat_fit(xd, yd, 4, 40, seed=5, early_stop=True)
    assert int(r["passes_skipped"].item()) > 0
    for k in ("assignments", "counts", "centroids"):
        assert torch.equal(r[k], full[k]), k
    for k in ("gamma", "beta"):
        torch.testing.assert_close(r[k], full[k], rtol=1e-5, atol=1e-6)
    torch.testing.assert_close(r["inertia"], full["inertia"], rtol=1e-12, atol=0)


@pytest.mark.parametrize("cap", [1, 64])
def test_with_short_changed_row_lists_and_given_initial_centroids(cap):
    """the length the decision reads counts every changed row, also those a workgroup appends to the device-wide
    list directly because its own list is full (forced by a tiny capacity); initial centroids given by the caller"""
    x, y = _mixture(1, 6007, 256, 8, 1.5, "f32")
    init = x[oracle.kmeanspp(x, 8, seed=3)]
    o = oracle.fit_early_stop(x, y, 8, 25, init_centroids=init.astype(np.float64))
    binding.select_path(binding.CAT_PATH_TILE)
    binding.debug_list_capacity(cap)
    try:
        r = cat_fit(dev_matrix(x, "f32"), dev_matrix(y, "f32"), 8, 25, early_stop=True,
                    init_centroids=torch.from_numpy(init).cuda())
    finally:
        binding.debug_list_capacity(0)
    assert (r["assignments"].cpu().numpy() == o["assignments"]).all()
    assert int(r["passes_skipped"].item()) == _expected_skips(int(o["stable_at"]), 25) > 0
    check_values(host_matrix(r["centroids"]), o["centroids"], RTOL["f32"], "centroids")
    np.testing.assert_allclose(r["inertia"].cpu().numpy(), o["inertia"], rtol=1e-4)


@pytest.mark.parametrize("D,path,padded", [(37, binding.CAT_PATH_AUTO, False), (37, binding.CAT_PATH_AUTO, True),
                                           (64, binding.CAT_PATH_STREAM, True)])
def test_shapes_outside_the_tile_kernels_run_every_pass(D, path, padded):
    """... unless the loop runs on a zero-padded copy of the rows (the default for rows that are not whole 16-byte
    groups), which stops like any loop of the tile kernels"""
    binding.select_path(path)
    x, y = _mixture(9, 1200, D, 3, 4.0, "f32")
    o = oracle.fit_early_stop(x, y, 3, 20, seed=1)
    assert 0 <= o["stable_at"] < 18
    binding.debug_padded_fit(padded)
    try:
        r = cat_fit(dev_matrix(x, "f32"), dev_matrix(y, "f32"), 3, 20, seed=1, early_stop=True)
    finally:
        binding.debug_padded_fit(True)
    on_copy = padded and path == binding.CAT_PATH_AUTO
    assert int(r["passes_skipped"].item()) == (_expected_skips(int(o["stable_at"]), 20) if on_copy else 0)
    assert (r["assignments"].cpu().numpy() == o["assignments"]).all()
    check_values(host_matrix(r["centroids"]), o["centroids"], RTOL["f32"], "centroids")
    np.testing.assert_allclose(r["inertia"].cpu().numpy(), o["inertia"], rtol=1e-4)


def test_captures_into_a_hip_graph_and_replays():
    """the decision to leave a pass out is taken on the device: captured once, every replay gives the eager result"""
    x, y = _mixture(0, 4096, 64, 4, 3.0, "f32")
    xd, yd = dev_matrix(x, "f32"), dev_matrix(y, "f32")
    ws = torch.empty(binding.cat_fit_workspace_bytes(4096, 64, 4), dtype=torch.uint8, device="cuda")

    def run():
        return cat_fit(xd, yd, 4, 30, seed=0, early_stop=True, workspace=ws)

    ref = {k: v.clone() for k, v in run().items()}
    assert int(ref["passes_skipped"].item()) > 0
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        r = run()
    for _ in range(3):
        for t in r.values():
            t.zero_()
        ws.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for k in ("assignments", "counts", "centroids", "passes_skipped"):
            assert torch.equal(r[k], ref[k]), k
        for k in ("gamma", "beta"):
            torch.testing.assert_close(r[k], ref[k], rtol=1e-5, atol=1e-6)
        torch.testing.assert_close(r["inertia"], ref["inertia"], rtol=1e-12, atol=0)
    # the same graph on other rows in the same buffers: one that settles a pass later, one that never does
    for seed, spread, skips in ((7, 0.8, 26), (5, 1.0, 0)):
        x2, y2 = _mixture(seed, 4096, 64, 4, spread, "f32")
        assert _expected_skips(int(oracle.fit_early_stop(x2, y2, 4, 30, seed=0)["stable_at"]), 30) == skips
        xd.copy_(torch.from_numpy(x2))
        yd.copy_(torch.from_numpy(y2))
        eager = {k: v.clone() for k, v in run().items()}
        for t in r.values():
            t.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert int(r["passes_skipped"].item()) == skips
        for k in ("assignments", "counts", "centroids", "passes_skipped"):
            assert torch.equal(r[k], eager[k]), k
        torch.testing.assert_close(r["inertia"], eager["inertia"], rtol=1e-12, atol=0)


def test_process_wide_switch_leaves_the_other_fits_unchanged():
    """best-of-several fit and the fit with the PCA front-end, with and without the switch: the integer outputs and
    the centroids bit for bit, the objectives to rounding; cat_fit itself too"""
    from paper_2509_26277_amd import cat_fit_pca, cat_fit_restarts
    x, y = _mixture(0, 4096, 64, 4, 3.0, "f32")
    xd, yd = dev_matrix(x, "f32"), dev_matrix(y, "f32")

    def runs():
        return (cat_fit_restarts(xd, yd, 4, 30, seed=2, restarts=3, seeding=binding.CAT_SEED_KMEANSPP),
                cat_fit_pca(xd, yd, 4, 8, 30, seed=2), cat_fit(xd, yd, 4, 30, seed=2))

    ref = runs()
    binding.allow_early_stop(True)
    try:
        got = runs()
    finally:
        binding.allow_early_stop(False)
    for which, (g, r) in enumerate(zip(got, ref)):
        for k, v in r.items():
            if v is None:
                continue
            # two PCA fits differ in the last bits (their covariance is summed with atomics): values to rounding there
            if k in ("gamma", "beta", "inertia", "final_inertia") or (which == 1 and v.dtype.is_floating_point):
                torch.testing.assert_close(g[k], v, rtol=1e-4, atol=1e-5)
            else:
                assert torch.equal(g[k], v), k


def test_bad_arguments_are_refused():
    x = torch.zeros((10, 4), device="cuda")
    lib = binding.load_library()
    ws = torch.empty(binding.cat_fit_workspace_bytes(10, 4, 2), dtype=torch.uint8, device="cuda")
    out = torch.empty((2, 4), device="cuda")
    a = torch.empty(10, dtype=torch.int32, device="cuda")
    rc = lib.cat_fit_early_stop(x.data_ptr(), x.data_ptr(), 10, 4, 2, 3, 0, binding.CAT_F32, None, out.data_ptr(),
                                out.data_ptr(), out.data_ptr(), a.data_ptr(), None, None, None, ws.data_ptr(),
                                ws.numel(), None)
    assert rc == 1 and b"passes_skipped" in lib.cat_last_error()
