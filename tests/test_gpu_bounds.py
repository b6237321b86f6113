"""GPU parity of the Lloyd loop that leaves rows out by distance bounds (cat_fit_bounds).

What defines the method is that it returns what the plain loop returns.  The library is compared with its own
cat_fit bit for bit and with the oracle's bound-based loop (``oracle.fit_bounds``, itself pinned to the plain loop)
to the usual tolerances.  The numbers of rows the two evaluate are not the same quantity (the oracle keeps Hamerly's
separate bounds and tightens them, the library keeps one gap per row and allows for the rounding of its scores), so
they are compared through what both must satisfy: every row that changes cluster in a pass is evaluated by it, and
a settled, separated mixture is not evaluated again."""
import numpy as np
import pytest
import torch

import oracle
from paper_2509_26277_amd import cat_fit, workloads
from paper_2509_26277_amd.binding import CAT_PATH_AUTO, CAT_PATH_STREAM, select_path

from parity_util import CENTROID_RTOL, RTOL, check_values, dev_matrix, host_matrix

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _auto_path_after():
    yield
    select_path(CAT_PATH_AUTO)


def _mixture(seed, N, D, C, dt, spread=2.0):
    rng = np.random.default_rng(seed)
    centres = rng.standard_normal((C, D)) * spread
    lab = rng.integers(0, C, N)
    y = (centres[lab] + rng.standard_normal((N, D))).astype(np.float32)
    x = (y * rng.uniform(0.6, 1.4, D).astype(np.float32) + 0.2 * rng.standard_normal((N, D)).astype(np.float32)).astype(np.float32)
    if dt == "bf16":
        x, y = workloads.round_to_bf16(x), workloads.round_to_bf16(y)
    return x, y


def _same_as_plain(b, p, iters):
    for key in ("centroids", "assignments", "counts"):
        assert torch.equal(b[key], p[key]), key
    for key in ("gamma", "beta"):  # (the statistics are summed with atomics: two runs agree to the last bits, not bit for bit)
        torch.testing.assert_close(b[key], p[key], rtol=1e-5, atol=1e-6)
    jb, jp = b["inertia"].cpu().numpy(), p["inertia"].cpu().numpy()
    full = [t for t in (0, 1, 2, iters) if t <= iters]
    np.testing.assert_allclose(jb[full], jp[full], rtol=5e-4)  # (the two may rank with different operand variants)


def _rows_that_change(x, K, iters, seed):
    cent = x[oracle.init_indices(len(x), K, seed)].astype(np.float64)
    prev, out = None, []
    for t in range(iters + 1):
        a = oracle.assign(x, cent)
        out.append(len(x) if prev is None else int((a != prev).sum()))
        if t < iters:
            cent, _ = oracle.update(x, a, cent)
        prev = a
    return out


@pytest.mark.parametrize("N,D,K,iters,dt,spread", [
    (6000, 64, 6, 12, "f32", 2.0),
    (5000, 136, 9, 10, "bf16", 2.0),
    (4099, 260, 40, 9, "f32", 0.7),      # overlapping components: rows keep moving
    (3000, 1000, 16, 8, "f32", 1.0),
    (2500, 2048, 64, 6, "bf16", 2.0),    # chunked operand
    (1500, 32, 5, 4, "f32", 2.0),        # one pass over listed rows
    (1500, 32, 5, 3, "f32", 2.0),        # too few iterations for any: the plain loop
    (900, 37, 4, 6, "f32", 2.0),         # rows that are not whole 16-byte groups: the loop runs on a zero-padded copy
    (2000, 16, 1, 6, "f32", 2.0),        # one cluster
    (3000, 260, 150, 6, "f32", 1.0),     # more than 128 clusters on long rows: two launches per pass, no bounds kept
    (3000, 64, 150, 6, "f32", 1.0),      # more than 128 clusters on short rows: one launch, bounds kept
])
def test_same_outputs_as_the_plain_loop_and_the_oracle(N, D, K, iters, dt, spread):
    x, y = _mixture(N + D + K, N, D, max(K, 2), dt, spread)
    xd, yd = dev_matrix(x, dt), dev_matrix(y, dt)
    b = cat_fit(xd, yd, K, iters, seed=7, bounds=True)
    _same_as_plain(b, cat_fit(xd, yd, K, iters, seed=7), iters)
    o = oracle.fit_bounds(x, y, K, iters, seed=7)
    assert (b["assignments"].cpu().numpy() == o["assignments"]).all()
    assert (b["counts"].cpu().numpy() == o["counts"]).all()
    check_values(host_matrix(b["centroids"]), o["centroids"], CENTROID_RTOL, "centroids")
    check_values(host_matrix(b["gamma"]), o["gamma"], RTOL[dt], "gamma")
    check_values(host_matrix(b["beta"]), o["beta"], RTOL[dt], "beta")
    ev = b["rows_evaluated"].cpu().numpy()
    assert ev.shape == (iters + 1,) and ev[0] == N and ev[-1] == N and (ev >= 0).all() and (ev <= N).all()
    assert (ev >= np.asarray(_rows_that_change(x, K, iters, 7))).all()  # a row that changes cluster was evaluated
    tile_shape = not (K > 128 and D > 128)
    if iters >= 4 and tile_shape:
        assert (ev[:3] == N).all()
        assert ev[3:-1].min() < N  # the bounds do leave rows out
        assert np.isnan(b["inertia"].cpu().numpy()[3:-1]).all()
    else:
        assert (ev == N).all()


def test_a_settled_separated_mixture_is_not_read_again():
    rng = np.random.default_rng(4)
    centres = rng.standard_normal((4, 64)) * 10.0
    lab = rng.integers(0, 4, 20000)
    x = (centres[lab] + rng.standard_normal((20000, 64))).astype(np.float32)
    init = torch.from_numpy((centres + 0.5).astype(np.float32)).cuda()
    y = (1.5 * x + 0.25 + 0.1 * rng.standard_normal(x.shape)).astype(np.float32)
    xd, yd = dev_matrix(x, "f32"), dev_matrix(y, "f32")
    b = cat_fit(xd, yd, 4, 10, init_centroids=init, bounds=True)
    assert (b["assignments"].cpu().numpy() == lab).all()
    ev = b["rows_evaluated"].cpu().numpy()
    assert ev[:3].tolist() == [20000] * 3 and ev[-1] == 20000
    assert (ev[3:-1] == 0).all()
    _same_as_plain(b, cat_fit(xd, yd, 4, 10, init_centroids=init), 10)


def test_duplicate_rows_empty_clusters_and_exact_ties():
    rng = np.random.default_rng(8)
    base = rng.integers(-3, 4, (6, 32)).astype(np.float32)
    x = np.repeat(base, 300, axis=0)
    y = (x * 1.5 + 0.25).astype(np.float32)
    xd, yd = dev_matrix(x, "f32"), dev_matrix(y, "f32")
    for K in (3, 9, 20):
        b = cat_fit(xd, yd, K, 6, seed=K, bounds=True)
        _same_as_plain(b, cat_fit(xd, yd, K, 6, seed=K), 6)
        o = oracle.fit_bounds(x, y, K, 6, seed=K)
        assert (b["assignments"].cpu().numpy() == o["assignments"]).all()
        assert (b["counts"].cpu().numpy() == o["counts"]).all()


def test_the_streaming_path_runs_the_plain_loop():
    x, y = _mixture(3, 2000, 64, 5, "f32")
    xd, yd = dev_matrix(x, "f32"), dev_matrix(y, "f32")
    select_path(CAT_PATH_STREAM)
    b = cat_fit(xd, yd, 5, 6, seed=1, bounds=True)
    assert (b["rows_evaluated"].cpu().numpy() == 2000).all()
    _same_as_plain(b, cat_fit(xd, yd, 5, 6, seed=1), 6)


@pytest.mark.parametrize("name", ["cfg2", "cfg3", "cfg4"])
def test_full_size_workloads(name):
    w = workloads.make(name)
    K, dt, iters = w["K"], w["dtype"], w["iters"]
    lq, fp = dev_matrix(w["lq"], dt), dev_matrix(w["fp"], dt)
    b = cat_fit(lq, fp, K, iters, seed=w["seed"], bounds=True)
    _same_as_plain(b, cat_fit(lq, fp, K, iters, seed=w["seed"]), iters)
    ev = b["rows_evaluated"].cpu().numpy()
    print(name, "rows evaluated per pass:", ev.tolist())
    assert ev[0] == w["N"] and ev[-1] == w["N"] and ev[3:-1].min() < w["N"]
