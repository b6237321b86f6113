"""The queue of rows whose exact re-rank is put off to the end of a workgroup's tiles (assignment passes of the tile
kernels without distance bounds).

Rows whose two best scores are within the error bound of the split arithmetic are queued in fast memory and measured in
double precision by all waves once the workgroup has no tiles left; a row that finds the queue full, or has more than
eight candidates, is measured where it is found.  The inputs here put a large share of the rows inside the bound (a
common offset makes |x||c| large against the gaps between scores; duplicated centroids make exact ties), and every
capacity (no queue, 1, 7, the default) must give the oracle's assignments, the same ones bit for bit, and the same
counts, objective, list of changed rows (seen through the centroids of the fused loop) and first rows."""
import numpy as np
import pytest
import torch

import oracle
from paper_2509_26277_amd import binding, cat_assign, cat_fit, workloads

from parity_util import CENTROID_RTOL, RTOL, check_assignments, check_values, dev_matrix, host_matrix

pytestmark = pytest.mark.gpu

CAPS = (-1, 1, 7, 0)


@pytest.fixture(autouse=True)
def _defaults_after():
    binding.select_path(binding.CAT_PATH_TILE)
    yield
    binding.debug_rerank_queue(0)
    binding.select_path(binding.CAT_PATH_AUTO)


def _crowded(seed, N, D, K, dt, offset, dup=0):
    """overlapping clusters far from the origin; the last `dup` centroids repeat the first ones (exact ties), or, with
    dup < 0, the last -dup all repeat centroid 0 (rows with 1 - dup candidates)"""
    rng = np.random.default_rng(seed)
    cent = (offset + 0.5 * rng.standard_normal((K, D))).astype(np.float32)
    if dup > 0:
        cent[K - dup:] = cent[:dup]
    elif dup < 0:
        cent[K + dup:] = cent[0]
    x = (cent[rng.integers(0, K, N)] + 0.7 * rng.standard_normal((N, D))).astype(np.float32)
    y = (1.3 * x + 0.1 * rng.standard_normal((N, D))).astype(np.float32)
    if dt == "bf16":
        x, y = workloads.round_to_bf16(x), workloads.round_to_bf16(y)
    return x, y, cent


@pytest.mark.parametrize("N,D,K,dt,offset,dup", [
    (5003, 64, 12, "f32", 40.0, 0),      # resident operand, one cluster tile
    (4100, 200, 40, "f32", 25.0, 3),     # three cluster tiles, three exact ties per row of those clusters
    (3000, 2048, 64, "bf16", 24.0, 2),   # the chunked operand: eight waves in lockstep
    (2500, 1000, 16, "f32", 30.0, 0),
    (1500, 96, 20, "f32", 10.0, -12),    # rows of cluster 0 have 13 candidates: measured on the spot
    (1200, 64, 150, "f32", 5.0, -149),   # every centroid the same: 150 candidates per row, sixteen cluster tiles
    (1000, 1000, 150, "f32", 3.0, -149), # the same with the clusters split over two launches
])
def test_single_pass_every_capacity(N, D, K, dt, offset, dup):
    x, _, cent = _crowded(N + D, N, D, K, dt, offset, dup)
    xd, cd = dev_matrix(x, dt), torch.from_numpy(cent).cuda()
    o_a, d1, d2 = oracle.assign(x, cent.astype(np.float64), want_distances=True)
    ref = None
    for cap in CAPS:
        binding.debug_rerank_queue(cap)
        a, counts, inertia = cat_assign(xd, cd)
        a_h = a.cpu().numpy()
        check_assignments(a_h, o_a, d1, d2, f"queue capacity {cap}")
        assert counts.cpu().numpy().tolist() == np.bincount(a_h, minlength=K).tolist()
        # (rows this far from the origin: the term of a row that is not re-ranked, |x|^2 + score in single precision,
        # carries the error bound of a score, a visible share of distances this small beside |x||c|)
        np.testing.assert_allclose(inertia.cpu().numpy()[0], d1.sum(), rtol=2e-2)
        if ref is None:
            ref, ref_inertia = a_h, inertia.cpu().numpy()[0]
        assert (a_h == ref).all(), cap
        np.testing.assert_allclose(inertia.cpu().numpy()[0], ref_inertia, rtol=1e-9)  # the same terms, another order
    if dup:  # the later copy of a repeated centroid never wins
        assert (ref < K - abs(dup)).all()


@pytest.mark.parametrize("N,D,K,dt,offset", [
    (6000, 72, 9, "f32", 30.0),
    (2300, 2048, 64, "bf16", 24.0),
    (4000, 520, 33, "f32", 20.0),
])
def test_fused_loop_every_capacity(N, D, K, dt, offset):
    x, y, _ = _crowded(7 * N + K, N, D, K, dt, offset)
    xd, yd = dev_matrix(x, dt), dev_matrix(y, dt)
    iters = 5
    o = oracle.fit(x, y, K, iters, seed=11)
    _, d1, d2 = oracle.assign(x, o["centroids"], want_distances=True)
    ref = None
    for cap in CAPS:
        binding.debug_rerank_queue(cap)
        r = cat_fit(xd, yd, K, iters, seed=11)
        a = r["assignments"].cpu().numpy()
        exempt = check_assignments(a, o["assignments"], d1, d2, f"queue capacity {cap}")
        assert r["counts"].cpu().numpy().tolist() == np.bincount(a, minlength=K).tolist()
        check_values(host_matrix(r["centroids"]), o["centroids"], RTOL[dt] if exempt else CENTROID_RTOL, f"capacity {cap} centroids")
        np.testing.assert_allclose(r["inertia"].cpu().numpy(), o["inertia"], rtol=2e-2)  # (see the single pass)
        if ref is None:
            ref = r
        else:
            np.testing.assert_allclose(r["inertia"].cpu().numpy(), ref["inertia"].cpu().numpy(), rtol=1e-9)
            assert torch.equal(r["assignments"], ref["assignments"]), cap
            assert torch.equal(r["counts"], ref["counts"]), cap
            torch.testing.assert_close(r["centroids"], ref["centroids"], rtol=1e-6, atol=1e-6)


def test_queue_and_short_changed_row_list_together():
    """queued rows that changed cluster join the list at the end of the workgroup's tiles, also when the list is full"""
    N, D, K = 5000, 64, 10
    x, y, _ = _crowded(5, N, D, K, "f32", 35.0)
    xd, yd = dev_matrix(x, "f32"), dev_matrix(y, "f32")
    binding.debug_rerank_queue(-1)
    ref = cat_fit(xd, yd, K, 6, seed=2)
    try:
        binding.debug_list_capacity(3)
        binding.debug_rerank_queue(0)
        r = cat_fit(xd, yd, K, 6, seed=2)
    finally:
        binding.debug_list_capacity(0)
    assert torch.equal(r["assignments"], ref["assignments"])
    assert torch.equal(r["counts"], ref["counts"])
    torch.testing.assert_close(r["centroids"], ref["centroids"], rtol=1e-6, atol=1e-6)


def test_hook_rejects_bad_values():
    for bad in (-2, 257):
        with pytest.raises(binding.CatError) as e:
            binding.debug_rerank_queue(bad)
        assert e.value.status == 1
