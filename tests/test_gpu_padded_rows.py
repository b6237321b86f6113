"""Fits of rows that are not a whole number of 16-byte groups (D not a multiple of 4, of 8 for bf16).

The matrix-core kernels do not take such rows as they lie; the fits copy them once into rows padded with zero channels
and run their Lloyd loops on the copy.  Zero channels change no distance, so everything must equal the oracle's fit of
the original rows to the usual bars, and the library's fit on the streaming kernels (the copy switched off) to
rounding; centroids, gamma and beta come back with D columns."""
import numpy as np
import pytest
import torch

import oracle
from paper_2509_26277_amd import binding, cat_fit, cat_fit_multi_k, cat_fit_restarts, workloads

from parity_util import CENTROID_RTOL, RTOL, check_assignments, check_values, dev_matrix, host_matrix

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _defaults_after():
    yield
    binding.debug_padded_fit(True)
    binding.select_path(binding.CAT_PATH_AUTO)


def _mixture(seed, N, D, C, dt, spread=2.0):
    rng = np.random.default_rng(seed)
    centres = rng.standard_normal((C, D)) * spread
    lab = rng.integers(0, C, N)
    y = (centres[lab] + rng.standard_normal((N, D))).astype(np.float32)
    x = (y * rng.uniform(0.6, 1.4, D).astype(np.float32) + 0.2 * rng.standard_normal((N, D)).astype(np.float32)).astype(np.float32)
    if dt == "bf16":
        x, y = workloads.round_to_bf16(x), workloads.round_to_bf16(y)
    return x, y


def _against_oracle(r, o, x, dt, what):
    _, d1, d2 = oracle.assign(x, o["centroids"], want_distances=True)
    a = r["assignments"].cpu().numpy()
    exempt = check_assignments(a, o["assignments"], d1, d2, what)
    assert r["counts"].cpu().numpy().tolist() == np.bincount(a, minlength=len(o["counts"])).tolist()
    check_values(host_matrix(r["centroids"]), o["centroids"], RTOL[dt] if exempt else CENTROID_RTOL, what + " centroids")
    if exempt == 0:
        check_values(host_matrix(r["gamma"]), o["gamma"], RTOL[dt], what + " gamma")
        check_values(host_matrix(r["beta"]), o["beta"], RTOL[dt], what + " beta")
    np.testing.assert_allclose(r["inertia"].cpu().numpy(), o["inertia"], rtol=1e-4)


@pytest.mark.parametrize("N,D,K,iters,dt", [
    (3000, 1001, 16, 5, "f32"),      # three channels of padding, chunked operand
    (2100, 1002, 16, 4, "bf16"),     # bf16 rows: padded to a multiple of 8
    (4099, 37, 9, 6, "f32"),         # rows not a multiple of the tile either
    (2500, 129, 33, 5, "f32"),
    (900, 30, 40, 4, "bf16"),
    (777, 7, 5, 6, "f32"),           # more padding than a quarter of the row
    (300, 1, 3, 5, "f32"),           # one channel
    (2000, 261, 200, 4, "f32"),      # more than 128 clusters: two launches per pass on the copy
    (1500, 61, 2, 2, "f32"),         # the fewest iterations that make a copy
])
def test_fit_on_the_copy_matches_the_oracle_and_the_streaming_kernels(N, D, K, iters, dt):
    x, y = _mixture(N + D + K, N, D, max(2, min(K, 9)), dt)
    xd, yd = dev_matrix(x, dt), dev_matrix(y, dt)
    r = cat_fit(xd, yd, K, iters, seed=3)
    assert r["centroids"].shape == (K, D) and r["gamma"].shape == (K, D)
    o = oracle.fit(x, y, K, iters, seed=3)
    _against_oracle(r, o, x, dt, f"{N}x{D} K={K} {dt}")
    binding.debug_padded_fit(False)
    s = cat_fit(xd, yd, K, iters, seed=3)
    if torch.equal(s["assignments"], r["assignments"]):
        assert torch.equal(s["counts"], r["counts"])
        torch.testing.assert_close(s["centroids"], r["centroids"], rtol=1e-5, atol=1e-6)
        torch.testing.assert_close(s["gamma"], r["gamma"], rtol=RTOL[dt], atol=RTOL[dt])
    else:  # a near-tie may fall either way between the two kernels: each must then be within the bars of the oracle
        _against_oracle(s, o, x, dt, "streaming kernels")


def test_the_copy_is_made_only_for_two_or_more_iterations_and_the_default_path():
    N, D, K = 2000, 203, 7
    x, y = _mixture(1, N, D, 7, "f32")
    xd, yd = dev_matrix(x, "f32"), dev_matrix(y, "f32")
    for iters, path in ((0, binding.CAT_PATH_AUTO), (1, binding.CAT_PATH_AUTO), (4, binding.CAT_PATH_STREAM)):
        binding.select_path(path)
        binding.debug_padded_fit(True)
        a = cat_fit(xd, yd, K, iters, seed=2)
        binding.debug_padded_fit(False)
        b = cat_fit(xd, yd, K, iters, seed=2)
        for key in ("centroids", "assignments", "counts"):  # the same kernels ran: bit for bit
            assert torch.equal(a[key], b[key]), (iters, path, key)
    # the scratch of a fit of such rows holds the copy; that of rows the tile kernels take as they lie does not
    assert binding.cat_fit_workspace_bytes(N, D, K) > binding.cat_fit_workspace_bytes(N, 204, K) + N * 204 * 4
    assert binding.cat_fit_workspace_bytes(N, 204, K) < N * 204 * 4
    binding.select_path(binding.CAT_PATH_TILE)  # a forced family is not quietly replaced
    with pytest.raises(binding.CatError):
        cat_fit(xd, yd, K, 4, seed=2)


def test_given_initial_centroids_bounds_and_early_stop():
    N, D, K, iters = 5000, 131, 6, 14
    x, y = _mixture(5, N, D, 6, "f32", spread=3.0)
    xd, yd = dev_matrix(x, "f32"), dev_matrix(y, "f32")
    rng = np.random.default_rng(0)
    init = np.ascontiguousarray(x[rng.choice(N, K, replace=False)])
    o = oracle.fit(x, y, K, iters, init_centroids=init.astype(np.float64))
    plain = cat_fit(xd, yd, K, iters, init_centroids=torch.from_numpy(init).cuda())
    _against_oracle(plain, o, x, "f32", "given initial centroids")
    b = cat_fit(xd, yd, K, iters, init_centroids=torch.from_numpy(init).cuda(), bounds=True)
    for key in ("centroids", "assignments", "counts"):
        assert torch.equal(b[key], plain[key]), key
    ev = b["rows_evaluated"].cpu().numpy()
    assert ev[0] == N and ev[-1] == N and ev[3:-1].min() < N  # the bounds are kept on the copy
    e = cat_fit(xd, yd, K, iters, init_centroids=torch.from_numpy(init).cuda(), early_stop=True)
    for key in ("centroids", "assignments", "counts"):
        assert torch.equal(e[key], plain[key]), key
    oe = oracle.fit_early_stop(x, y, K, iters, init_centroids=init.astype(np.float64))
    if oe["stable_at"] >= 0:
        assert int(e["passes_skipped"].item()) == max(0, iters - 1 - max(int(oe["stable_at"]), 2))


def test_restarts_and_a_grid_of_cluster_counts_run_on_the_copy():
    N, D, iters = 3000, 75, 5
    x, y = _mixture(8, N, D, 8, "f32")
    xd, yd = dev_matrix(x, "f32"), dev_matrix(y, "f32")
    r = cat_fit_restarts(xd, yd, 8, iters, seed=20, restarts=4)
    single = cat_fit(xd, yd, 8, iters, seed=20 + int(r["best_run"]))
    for key in ("centroids", "assignments", "counts"):
        assert torch.equal(r[key], single[key]), key
    o = oracle.fit_restarts(x, y, 8, iters, seed=20, restarts=4)
    np.testing.assert_allclose(r["final_inertia"].cpu().numpy(), o["final_inertia"], rtol=1e-4)
    Ks = [3, 20, 300, 8]  # 300: outside the tile kernels at any row length, runs on the original rows
    m = cat_fit_multi_k(xd, yd, Ks, iters, seed=4)
    om = oracle.fit_multi_k(x, y, Ks, iters, seed=4)
    for K, e, oe in zip(Ks, m, om):
        s = cat_fit(xd, yd, K, iters, seed=4)
        for key in ("centroids", "assignments", "counts"):
            assert torch.equal(e[key], s[key]), (K, key)
        _against_oracle(e, oe, x, "f32", f"K={K} of the list")


def test_captures_into_a_hip_graph_and_replays():
    N, D, K, iters = 4000, 203, 5, 6
    x, y = _mixture(2, N, D, 5, "f32")
    xd, yd = dev_matrix(x, "f32"), dev_matrix(y, "f32")
    ws = torch.empty(binding.cat_fit_workspace_bytes(N, D, K), dtype=torch.uint8, device="cuda")

    def run():
        return cat_fit(xd, yd, K, iters, seed=1, workspace=ws)

    ref = {k: v.clone() for k, v in run().items()}
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
        for key in ("centroids", "assignments", "counts"):
            assert torch.equal(r[key], ref[key]), key
        torch.testing.assert_close(r["gamma"], ref["gamma"], rtol=1e-5, atol=1e-6)
        torch.testing.assert_close(r["beta"], ref["beta"], rtol=1e-5, atol=1e-6)
