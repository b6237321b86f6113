"""GPU-vs-oracle parity of the CAT hot path, through the C ABI.

Step level ("teacher forced": the oracle's state is fed to one GPU step) and end
to end, on structure-preserving small copies of the five workloads and on the
method's edge cases.  Sizes span several 16-row tiles plus a ragged tail and the
oracle finishes each in seconds.  Both kernel families are covered where a shape
fits the tile kernels.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2509_26277_amd import binding, workloads
from paper_2509_26277_amd import cat_apply, cat_assign, cat_fit, cat_stats, cat_update

from parity_util import (CENTROID_RTOL, RTOL, check_assignments, check_values, dev_matrix, f32_round, host_matrix)

pytestmark = pytest.mark.gpu

# every shape below that is parametrised over PATHS fits the tile kernels, so the second entry
# really runs them (a forced path that does not fit returns CAT_ERR_UNSUPPORTED)
PATHS = [binding.CAT_PATH_STREAM, binding.CAT_PATH_TILE]


@pytest.fixture(autouse=True)
def _auto_path_after():
    yield
    binding.select_path(binding.CAT_PATH_AUTO)


def small(name, n_rows):
    return workloads.make(name, n_rows=n_rows)


SMALL_FIT = [("cfg1", 4096), ("cfg2", 1531), ("cfg3", 6007), ("cfg4", 1100)]


# ---------------------------------------------------------------------------
# seeded init
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("name,n", [("cfg1", 4096), ("cfg4", 700)])
def test_seeded_init_rows_are_copied_exactly(name, n):
    w = small(name, n)
    lq = dev_matrix(w["lq"], w["dtype"])
    fp = dev_matrix(w["fp"], w["dtype"])
    r = cat_fit(lq, fp, w["K"], iters=0, seed=4242)
    idx = oracle.init_indices(n, w["K"], 4242)
    assert (host_matrix(r["centroids"]) == w["lq"][idx].astype(np.float64)).all()


# ---------------------------------------------------------------------------
# teacher-forced steps
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("path", PATHS)
@pytest.mark.parametrize("name,n", SMALL_FIT)
def test_assign_step(name, n, path):
    binding.select_path(path)
    w = small(name, n)
    K = w["K"]
    # the oracle's centroids after 2 iterations, rounded to the float the GPU is handed
    o = oracle.fit(w["lq"], w["fp"], K, iters=2, seed=w["seed"])
    cent = f32_round(o["centroids"])
    a_o, d1, d2 = oracle.assign(w["lq"], cent, want_distances=True)
    a_g, counts, inertia = cat_assign(dev_matrix(w["lq"], w["dtype"]), torch.from_numpy(cent.astype(np.float32)).cuda())
    check_assignments(a_g.cpu().numpy(), a_o, d1, d2, f"{name} assign")
    assert counts.cpu().numpy().tolist() == np.bincount(a_g.cpu().numpy(), minlength=K).tolist()
    assert inertia.item() == pytest.approx(d1.sum(), rel=1e-4)


@pytest.mark.parametrize("path", PATHS)
@pytest.mark.parametrize("name,n", SMALL_FIT)
def test_update_and_stats_steps(name, n, path):
    # the forced tile path also takes the segmented sums over cluster-ordered rows on every shape
    binding.select_path(path)
    w = small(name, n)
    K, dt = w["K"], w["dtype"]
    o = oracle.fit(w["lq"], w["fp"], K, iters=3, seed=w["seed"])
    a = o["assignments"]
    lq, fp = dev_matrix(w["lq"], dt), dev_matrix(w["fp"], dt)
    a_dev = torch.from_numpy(a).cuda()
    prev = f32_round(o["centroids"]) + 0.25
    c_o, n_o = oracle.update(w["lq"], a, prev)
    c_g, n_g = cat_update(lq, a_dev, torch.from_numpy(prev.astype(np.float32)).cuda())
    assert n_g.cpu().numpy().tolist() == n_o.tolist()
    check_values(host_matrix(c_g), c_o, CENTROID_RTOL, f"{name} update")
    g_o, b_o, _ = oracle.affine(w["lq"], w["fp"], a, K)
    for hint in (None, c_g):
        g_g, b_g, n2 = cat_stats(lq, fp, a_dev, K, centroids=hint)
        assert n2.cpu().numpy().tolist() == n_o.tolist()
        check_values(host_matrix(g_g), g_o, RTOL[dt], f"{name} gamma")
        check_values(host_matrix(b_g), b_o, RTOL[dt], f"{name} beta")


# ---------------------------------------------------------------------------
# end to end
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("path", PATHS)
@pytest.mark.parametrize("name,n", SMALL_FIT)
def test_fit_end_to_end(name, n, path):
    binding.select_path(path)
    w = small(name, n)
    K, dt, iters = w["K"], w["dtype"], min(w["iters"], 8)
    lq, fp = dev_matrix(w["lq"], dt), dev_matrix(w["fp"], dt)
    r = cat_fit(lq, fp, K, iters, seed=w["seed"])
    o = oracle.fit(w["lq"], w["fp"], K, iters, seed=w["seed"])
    _, d1, d2 = oracle.assign(w["lq"], o["centroids"], want_distances=True)
    a_g = r["assignments"].cpu().numpy()
    exempt = check_assignments(a_g, o["assignments"], d1, d2, f"{name} fit")
    assert r["counts"].cpu().numpy().tolist() == np.bincount(a_g, minlength=K).tolist()
    check_values(host_matrix(r["centroids"]), o["centroids"], RTOL[dt] if exempt else CENTROID_RTOL, f"{name} centroids")
    check_values(host_matrix(r["gamma"]), o["gamma"], RTOL[dt], f"{name} gamma")
    check_values(host_matrix(r["beta"]), o["beta"], RTOL[dt], f"{name} beta")
    np.testing.assert_allclose(r["inertia"].cpu().numpy(), o["inertia"], rtol=1e-4)
    # fit <-> apply: inference on the fitting rows reproduces the partition
    out, a2 = cat_apply(lq, r["centroids"], r["gamma"], r["beta"])
    same = (a2.cpu().numpy() == a_g)
    _, e1, e2 = oracle.assign(w["lq"], host_matrix(r["centroids"]), want_distances=True)
    assert ((e2 - e1)[~same] <= 1e-5 * e2[~same]).all()


@pytest.mark.parametrize("cap", [1, 5, 64])
@pytest.mark.parametrize("name,n", [("cfg1", 4096), ("cfg3", 6007), ("cfg4", 1100)])
def test_fit_with_short_changed_row_lists(name, n, cap):
    """The fused Lloyd loop when a workgroup's list of changed rows overflows (forced by a tiny capacity):
    the overflowing tiles append to the device-wide list directly.  Same results as ever."""
    binding.select_path(binding.CAT_PATH_TILE)
    binding.debug_list_capacity(cap)
    try:
        w = small(name, n)
        K, dt, iters = w["K"], w["dtype"], 6
        r = cat_fit(dev_matrix(w["lq"], dt), dev_matrix(w["fp"], dt), K, iters, seed=w["seed"])
    finally:
        binding.debug_list_capacity(0)
    o = oracle.fit(w["lq"], w["fp"], K, iters, seed=w["seed"])
    _, d1, d2 = oracle.assign(w["lq"], o["centroids"], want_distances=True)
    a_g = r["assignments"].cpu().numpy()
    exempt = check_assignments(a_g, o["assignments"], d1, d2, f"{name} fit")
    assert r["counts"].cpu().numpy().tolist() == np.bincount(a_g, minlength=K).tolist()
    check_values(host_matrix(r["centroids"]), o["centroids"], RTOL[dt] if exempt else CENTROID_RTOL, f"{name} centroids")
    check_values(host_matrix(r["gamma"]), o["gamma"], RTOL[dt], f"{name} gamma")
    np.testing.assert_allclose(r["inertia"].cpu().numpy(), o["inertia"], rtol=1e-4)


def test_list_capacity_hook_rejects_bad_values():
    for bad in (-1, 1025):
        with pytest.raises(binding.CatError) as e:
            binding.debug_list_capacity(bad)
        assert e.value.status == 1
    binding.debug_list_capacity(0)


@pytest.mark.parametrize("path", PATHS)
@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_update_and_stats_skip_rows_with_labels_outside_the_range(dt, path):
    """cat_update / cat_stats on caller-made assignments: a label outside [0, K) leaves the row out."""
    binding.select_path(path)
    rng = np.random.default_rng(77)
    N, D, K = 3001, 72, 5
    lq = rng.standard_normal((N, D)).astype(np.float32)
    fp = (1.1 * lq + 0.05 * rng.standard_normal((N, D))).astype(np.float32)
    if dt == "bf16":
        lq, fp = workloads.round_to_bf16(lq), workloads.round_to_bf16(fp)
    a = rng.integers(0, K, N).astype(np.int32)
    a[rng.random(N) < 0.1] = -1
    a[rng.random(N) < 0.05] = K
    a[a == 3] = 1  # and one empty cluster
    keep = (a >= 0) & (a < K)
    prev = rng.standard_normal((K, D)).astype(np.float32)
    c_o, n_o = oracle.update(lq[keep], a[keep], prev)
    g_o, b_o, _ = oracle.affine(lq[keep], fp[keep], a[keep], K)
    lq_d, fp_d, a_d = dev_matrix(lq, dt), dev_matrix(fp, dt), torch.from_numpy(a).cuda()
    c_g, n_g = cat_update(lq_d, a_d, torch.from_numpy(prev).cuda())
    assert n_g.cpu().numpy().tolist() == n_o.tolist()
    check_values(host_matrix(c_g), c_o, CENTROID_RTOL, "update")
    g_g, b_g, n2 = cat_stats(lq_d, fp_d, a_d, K)
    assert n2.cpu().numpy().tolist() == n_o.tolist()
    check_values(host_matrix(g_g), g_o, RTOL[dt], "gamma")
    check_values(host_matrix(b_g), b_o, RTOL[dt], "beta")


@pytest.mark.parametrize("path", PATHS)
@pytest.mark.parametrize("alpha", [1.0, 0.5, 0.0])
def test_apply_end_to_end(alpha, path):
    binding.select_path(path)
    w = small("cfg5", 3001)
    lq = dev_matrix(w["lq"], "f32")
    args = [torch.from_numpy(w[k]).cuda() for k in ("centroids", "gamma", "beta")]
    out, a = cat_apply(lq, *args, alpha=alpha)
    o_out, o_a = oracle.apply(w["lq"], w["centroids"], w["gamma"], w["beta"], alpha=alpha)
    _, d1, d2 = oracle.assign(w["lq"], w["centroids"].astype(np.float64), want_distances=True)
    check_assignments(a.cpu().numpy(), o_a, d1, d2, "cfg5 apply")
    ok = a.cpu().numpy() == o_a
    check_values(host_matrix(out)[ok], o_out[ok], RTOL["f32"], f"cfg5 corrected alpha={alpha}")
    if alpha == 0.0:
        assert (out == lq).all()


@pytest.mark.parametrize("path", PATHS)
def test_apply_bf16_rows(path):
    binding.select_path(path)
    w = small("cfg4", 900)
    K, D = w["K"], w["D"]
    rng = np.random.default_rng(5)
    cent = w["lq"][rng.choice(900, K, replace=False)]
    gamma = rng.uniform(0.8, 1.2, (K, D)).astype(np.float32)
    beta = rng.standard_normal((K, D)).astype(np.float32) * 0.3
    out, a = cat_apply(dev_matrix(w["lq"], "bf16"), *[torch.from_numpy(v).cuda() for v in (cent, gamma, beta)])
    o_out, o_a = oracle.apply(w["lq"], cent, gamma, beta)
    _, d1, d2 = oracle.assign(w["lq"], cent.astype(np.float64), want_distances=True)
    check_assignments(a.cpu().numpy(), o_a, d1, d2, "bf16 apply")
    ok = a.cpu().numpy() == o_a
    assert out.dtype == torch.bfloat16
    check_values(host_matrix(out)[ok], o_out[ok], RTOL["bf16"], "bf16 corrected")


# ---------------------------------------------------------------------------
# edge cases of the method
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("path", PATHS)
def test_ties_duplicates_and_midpoints_go_to_the_lowest_index(path):
    binding.select_path(path)
    rng = np.random.default_rng(3)
    D = 40
    base = np.round(rng.standard_normal((3, D)) * 4) / 2            # half-integers: exact arithmetic
    cent = np.stack([base[0], base[1], base[1], base[2], base[0]])  # duplicates 1==2, 0==4
    rows = [base[1], base[0], (base[1] + base[2]) / 2, (base[0] + base[2]) / 2]
    rows += [base[i % 3] + np.round(rng.standard_normal(D) * 2) / 4 for i in range(60)]
    lq = np.stack(rows).astype(np.float32)
    a_o, d1, d2 = oracle.assign(lq, cent, want_distances=True)
    assert a_o[:4].tolist() == [1, 0, 1, 0]
    a_g, _, _ = cat_assign(torch.from_numpy(lq).cuda(), torch.from_numpy(cent.astype(np.float32)).cuda())
    assert a_g.cpu().numpy().tolist() == a_o.tolist()     # exact ties included: no exemption here


@pytest.mark.parametrize("path", PATHS)
def test_empty_cluster_constant_channel_single_row(path):
    binding.select_path(path)
    w = small("cfg1", 500)
    lq_h = w["lq"].copy()
    fp_h = w["fp"].copy()
    lq_h[:, 3] = np.float32(0.1)          # a channel that is constant everywhere
    lq_h[499] = 50.0                      # one far row: a single-member cluster
    lq_h[499, 3] = np.float32(0.1)
    init = np.stack([lq_h[0], lq_h[1], np.full(64, -300.0, np.float32), lq_h[499]])  # cluster 2 stays empty
    r = cat_fit(torch.from_numpy(lq_h).cuda(), torch.from_numpy(fp_h).cuda(), 4, iters=4,
                init_centroids=torch.from_numpy(init).cuda())
    o = oracle.fit(lq_h, fp_h, 4, iters=4, init_centroids=init.astype(np.float64))
    assert o["counts"][2] == 0 and o["counts"][3] == 1
    assert (r["assignments"].cpu().numpy() == o["assignments"]).all()
    assert r["counts"].cpu().numpy().tolist() == o["counts"].tolist()
    g, b, c = host_matrix(r["gamma"]), host_matrix(r["beta"]), host_matrix(r["centroids"])
    assert (g[2] == 1.0).all() and (b[2] == 0.0).all() and (c[2] == -300.0).all()
    assert (g[3] == 0.0).all() and (b[3] == fp_h[499].astype(np.float64)).all()
    check_values(g, o["gamma"], 1e-4, "gamma")
    check_values(b, o["beta"], 1e-4, "beta")
    assert np.abs(g[:2, 3]).max() < 1e-4  # constant channel: gamma 0, beta = mean FP
    check_values(c, o["centroids"], 1e-4, "centroids")


# (N, D, K, path): odd D only runs on the streaming kernels; D % 4 == 0 on both; K = 200 and 256 use the
# widest cluster tiling of the tile kernel
DEGENERATE = [(1, 1, 1, 1), (7, 1, 7, 1), (65, 3, 2, 1), (200, 130, 1, 1), (333, 257, 19, 1),
              (1, 4, 1, 2), (9, 4, 9, 2), (65, 8, 2, 2), (200, 132, 1, 2), (333, 260, 19, 2), (700, 64, 200, 2),
              (1200, 36, 256, 2), (65, 8, 2, 0), (333, 257, 19, 0)]


@pytest.mark.parametrize("N,D,K,path", DEGENERATE)
def test_degenerate_shapes(N, D, K, path):
    binding.select_path(path)
    rng = np.random.default_rng(N * 1000 + D)
    lq = rng.standard_normal((N, D)).astype(np.float32)
    fp = (lq * 0.9 + 0.1 * rng.standard_normal((N, D))).astype(np.float32)
    r = cat_fit(torch.from_numpy(lq).cuda(), torch.from_numpy(fp).cuda(), K, iters=3, seed=11)
    o = oracle.fit(lq, fp, K, iters=3, seed=11)
    _, d1, d2 = oracle.assign(lq, o["centroids"], want_distances=True)
    check_assignments(r["assignments"].cpu().numpy(), o["assignments"], d1, d2, "degenerate")
    check_values(host_matrix(r["centroids"]), o["centroids"], 1e-4, "centroids")
    check_values(host_matrix(r["gamma"]), o["gamma"], 1e-4, "gamma")
    check_values(host_matrix(r["beta"]), o["beta"], 1e-4, "beta")
    out, a = cat_apply(torch.from_numpy(lq).cuda(), r["centroids"], r["gamma"], r["beta"], alpha=0.7)
    o_out, o_a = oracle.apply(lq, host_matrix(r["centroids"]), host_matrix(r["gamma"]), host_matrix(r["beta"]), 0.7)
    _, e1, e2 = oracle.assign(lq, host_matrix(r["centroids"]), want_distances=True)
    check_assignments(a.cpu().numpy(), o_a, e1, e2, "degenerate, inference")
    ok = a.cpu().numpy() == o_a
    check_values(host_matrix(out)[ok], o_out[ok], 1e-4, "corrected")


def test_forced_tile_path_reports_shapes_it_cannot_run():
    binding.select_path(binding.CAT_PATH_TILE)
    lq = torch.zeros((64, 7), device="cuda")  # odd D: rows are not 16-byte aligned
    with pytest.raises(binding.CatError) as e:
        cat_assign(lq, lq[:4].contiguous())
    assert e.value.status == 2
    with pytest.raises(binding.CatError) as e:
        cat_fit(lq, lq.clone(), 4, iters=1)
    assert e.value.status == 2


def test_device_errors_are_statuses_not_crashes():
    lq = torch.zeros((64, 8), device="cuda")
    with pytest.raises(binding.CatError) as e:
        cat_fit(lq, lq.clone(), 4, iters=1, workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert e.value.status == 3
    with pytest.raises(binding.CatError):
        cat_apply(lq, lq[:4].contiguous(), lq[:4].contiguous(), lq[:4].contiguous(), out=lq)


def test_whole_path_captures_into_a_hip_graph_and_replays():
    """Nothing on the path allocates, synchronises or uses a memset node, so cat_fit + cat_apply can be
    captured once and replayed; every replay (with eager work in between) reproduces the eager result."""
    w = small("cfg1", 4096)
    K, iters = w["K"], 6
    lq, fp = dev_matrix(w["lq"], "f32"), dev_matrix(w["fp"], "f32")
    ws = torch.empty(binding.cat_fit_workspace_bytes(4096, w["D"], K, binding.CAT_F32), dtype=torch.uint8, device="cuda")
    ws2 = torch.empty(max(256, binding.cat_apply_workspace_bytes(4096, w["D"], K, binding.CAT_F32)), dtype=torch.uint8,
                      device="cuda")
    out = torch.empty_like(lq)

    def run():
        r = cat_fit(lq, fp, K, iters, seed=5, workspace=ws)
        o, a = cat_apply(lq, r["centroids"], r["gamma"], r["beta"], alpha=0.5, out=out, workspace=ws2)
        return r, o, a

    r0, o0, a0 = run()
    ref = {k: v.clone() for k, v in r0.items()}
    o_ref, a_ref = o0.clone(), a0.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):  # warm-up on the capture stream's side, as torch asks for
        run()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        r, o, a = run()
    for _ in range(3):
        for t in (r["centroids"], r["gamma"], r["beta"], r["assignments"], r["counts"], o, a):
            t.zero_()  # eager work between replays; also proves the replay rewrites every output
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(r["assignments"], ref["assignments"]) and torch.equal(a, a_ref)
        assert torch.equal(r["counts"], ref["counts"])
        for k in ("centroids", "gamma", "beta"):
            torch.testing.assert_close(r[k], ref[k], rtol=1e-6, atol=1e-7)
        torch.testing.assert_close(o, o_ref, rtol=1e-6, atol=1e-6)
        torch.testing.assert_close(r["inertia"], ref["inertia"], rtol=1e-9, atol=0)
