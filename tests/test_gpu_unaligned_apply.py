"""CAT Inferencing on rows that are not a whole number of 16-byte groups (D not a multiple of 4, of 8 for bf16), through
the row-tile inference kernel's word-by-word instances: every row is still read once and ranked on the matrix cores.

Against the oracle to the usual bars (assignments identical except rows whose top-2 gap is below 1e-5 relative, values
within 1e-4 / 2e-2), and against the LDS streaming kernel, which took these shapes before and still takes the ones the
row-tile kernel has no instance for."""
import numpy as np
import pytest
import torch

import oracle
from paper_2509_26277_amd import binding, cat_apply, cat_apply_lp, cat_params_to_bf16, workloads

from parity_util import RTOL, check_assignments_lazy, check_values, dev_matrix, host_matrix

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _defaults_after():
    yield
    binding.debug_apply_kernel(0)
    binding.select_path(binding.CAT_PATH_AUTO)


def _problem(seed, N, D, K, dt):
    rng = np.random.default_rng(seed)
    comps = max(2, min(K, 9))
    mu = 2.0 * rng.standard_normal((comps, D))
    x = (mu[rng.integers(0, comps, N)] + rng.standard_normal((N, D))).astype(np.float32)
    if dt == "bf16":
        x = workloads.round_to_bf16(x)
    cent = x[rng.choice(N, K, replace=False)].astype(np.float32) + (0.05 * rng.standard_normal((K, D))).astype(np.float32)
    if K > 3:
        cent[K - 1] = cent[1]  # an exact tie between two clusters: the lower index wins
    gamma = rng.uniform(0.7, 1.3, (K, D)).astype(np.float32)
    beta = (0.3 * rng.standard_normal((K, D))).astype(np.float32)
    return x, cent, gamma, beta


SHAPES = [
    (3000, 1001, 16, "f32"),    # four vectors per lane and row, the last one holds a single channel in one lane
    (2500, 129, 33, "f32"),
    (1500, 61, 70, "f32"),
    (4099, 37, 9, "f32"),       # rows not a multiple of the tile either
    (777, 7, 5, "f32"),
    (1000, 5, 3, "f32"),        # one whole group and one word
    (800, 509, 100, "f32"),     # the one-part instance (K <= 128, more than 256 channels)
    (800, 255, 128, "f32"),
    (900, 6, 2, "f32"),
    (2100, 1002, 16, "bf16"),
    (900, 30, 40, "bf16"),
    (700, 10, 3, "bf16"),       # one whole group and one word of two channels
    (600, 1022, 20, "bf16"),
    (500, 3, 2, "f32"), (300, 1, 2, "f32"), (400, 6, 3, "bf16"), (256, 2, 2, "bf16"),   # rows shorter than a group
]


@pytest.mark.parametrize("N,D,K,dt", SHAPES)
def test_apply_matches_the_oracle_and_the_streaming_kernel(N, D, K, dt):
    x, cent, gamma, beta = _problem(N + D + K, N, D, K, dt)
    xd = dev_matrix(x, dt)
    f = lambda a: torch.from_numpy(a).cuda()
    binding.debug_apply_kernel(2)  # the row-tile kernel or an error: these shapes must have an instance
    for alpha in (1.0, 0.6):
        out, a = cat_apply(xd, f(cent), f(gamma), f(beta), alpha=alpha)
        o_out, o_a = oracle.apply(x, cent, gamma, beta, alpha)
        a = a.cpu().numpy()
        check_assignments_lazy(a, o_a, x, cent.astype(np.float64), f"{N}x{D} K={K} {dt}")
        if K > 3:
            assert not (a == K - 1).any()
        same = a == o_a
        check_values(host_matrix(out)[same], o_out[same], RTOL[dt], "corrected")
    out_b, _ = cat_apply(xd, f(cent), f(gamma), f(beta), alpha=0.6, want_assignments=False)
    assert torch.equal(out_b, out)
    binding.debug_apply_kernel(1)  # the LDS streaming kernel on the same call
    out_s, a_s = cat_apply(xd, f(cent), f(gamma), f(beta), alpha=0.6)
    agree = a_s.cpu().numpy() == a
    assert agree.mean() > 0.99
    check_values(host_matrix(out_s)[agree], host_matrix(out)[agree], RTOL[dt], "the two kernels")


def test_every_word_of_the_output_is_written_and_nothing_else():
    """the output sits inside a larger buffer filled with a marker: the rows are written whole, the words before
    and after them stay"""
    N, D, K = 1234, 1001, 8
    x, cent, gamma, beta = _problem(5, N, D, K, "f32")
    f = lambda a: torch.from_numpy(a).cuda()
    big = torch.full((N * D + 64,), float("nan"), device="cuda")
    out = big[32:32 + N * D].view(N, D)
    assert out.data_ptr() % 16 == 0
    cat_apply(dev_matrix(x, "f32"), f(cent), f(gamma), f(beta), out=out)
    assert torch.isnan(big[:32]).all() and torch.isnan(big[32 + N * D:]).all()
    assert not torch.isnan(out).any()
    o_out, _ = oracle.apply(x, cent, gamma, beta, 1.0)
    check_values(host_matrix(out), o_out, 1e-3, "corrected")  # (labels of near-ties aside: covered above)


@pytest.mark.parametrize("N,D,K", [(3000, 1001, 16), (2000, 37, 9), (1500, 255, 32)])
def test_bf16_output_and_bf16_parameters(N, D, K):
    """fp32 rows, parameters stored in bfloat16, corrected rows written as bfloat16: odd row lengths leave the output
    rows 2-byte aligned, so they are written one channel at a time"""
    x, cent, gamma, beta = _problem(N + D, N, D, K, "f32")
    f = lambda a: torch.from_numpy(a).cuda()
    cq, gq, bq = cat_params_to_bf16(f(cent)), cat_params_to_bf16(f(gamma)), cat_params_to_bf16(f(beta))
    big = torch.zeros((N * D + 16,), dtype=torch.bfloat16, device="cuda")
    big[:] = 7.0
    out = big[8:8 + N * D].view(N, D)
    out16, a16 = cat_apply_lp(dev_matrix(x, "f32"), cq, gq, bq, alpha=0.6, bf16_out=True, out=out)
    assert (big[:8] == 7.0).all() and (big[8 + N * D:] == 7.0).all()
    o16, oa16, (ocq, _, _) = oracle.apply_lp(x, cent, gamma, beta, alpha=0.6)
    a16 = a16.cpu().numpy()
    check_assignments_lazy(a16, oa16, x, ocq, "cat_apply_lp")
    check_values(host_matrix(out16)[a16 == oa16], o16[a16 == oa16], RTOL["bf16"], "corrected, low precision")


def test_long_launch_with_tiles_handed_out_in_order():
    N, D, K = 600000, 37, 9
    x, cent, gamma, beta = _problem(77, N, D, K, "f32")
    f = lambda a: torch.from_numpy(a).cuda()
    out, a = cat_apply(dev_matrix(x, "f32"), f(cent), f(gamma), f(beta), alpha=0.8)
    o_out, o_a = oracle.apply(x, cent, gamma, beta, 0.8)
    a = a.cpu().numpy()
    check_assignments_lazy(a, o_a, x, cent.astype(np.float64), "long launch")
    same = a == o_a
    check_values(host_matrix(out)[same], o_out[same], RTOL["f32"], "corrected")


def test_shapes_without_an_instance_still_take_the_streaming_kernel():
    # more than 256 clusters; the instance for 33 .. 64 clusters on rows of 2 .. 4 KB has no word-by-word form; bf16 rows
    # of more than 2 KB
    for N, D, K, dt in [(1200, 50, 300, "f32"), (900, 1001, 40, "f32"), (500, 1030, 8, "bf16")]:
        x, cent, gamma, beta = _problem(D + K, N, D, K, dt)
        f = lambda a: torch.from_numpy(a).cuda()
        with pytest.raises(binding.CatError):
            binding.debug_apply_kernel(2)
            cat_apply(dev_matrix(x, dt), f(cent), f(gamma), f(beta))
        binding.debug_apply_kernel(0)
        out, a = cat_apply(dev_matrix(x, dt), f(cent), f(gamma), f(beta))
        o_out, o_a = oracle.apply(x, cent, gamma, beta, 1.0)
        a = a.cpu().numpy()
        check_assignments_lazy(a, o_a, x, cent.astype(np.float64), "streaming kernel")
        check_values(host_matrix(out)[a == o_a], o_out[a == o_a], RTOL[dt], "corrected")


@pytest.mark.parametrize("N,D,K,dt", [(3000, 1001, 16, "f32"), (4099, 37, 9, "f32"), (800, 255, 128, "f32"), (2100, 1002, 16, "bf16"),
                                      (300, 1, 2, "f32")])
def test_assignment_step_without_the_map(N, D, K, dt):
    """cat_assign on these shapes: the same kernel with nothing stored but the labels, counts from the labels, the
    objective from the kernel's own scores (exact distances where it re-ranked)"""
    from paper_2509_26277_amd import cat_assign, cat_fit
    x, cent, _, _ = _problem(N + D, N, D, K, dt)
    xd = dev_matrix(x, dt)
    a, counts, inertia = cat_assign(xd, torch.from_numpy(cent).cuda())
    o_a, d1, _ = oracle.assign(x, cent.astype(np.float64), want_distances=True)
    a = a.cpu().numpy()
    check_assignments_lazy(a, o_a, x, cent.astype(np.float64), "cat_assign")
    assert counts.cpu().numpy().tolist() == np.bincount(a, minlength=K).tolist()
    assert float(inertia) == pytest.approx(d1.sum(), rel=1e-4)
    binding.debug_apply_kernel(1)  # the LDS streaming kernel
    a_s, c_s, i_s = cat_assign(xd, torch.from_numpy(cent).cuda())
    assert (a_s.cpu().numpy() == a).mean() > 0.99
    assert float(i_s) == pytest.approx(float(inertia), rel=1e-4)
    binding.debug_apply_kernel(0)
    # a fit too short for a padded copy of the rows runs its passes through the same step
    y = (1.2 * x + 0.1).astype(np.float32)
    if dt == "bf16":
        y = workloads.round_to_bf16(y)
    r = cat_fit(xd, dev_matrix(y, dt), K, 1, seed=3)
    o = oracle.fit(x, y, K, 1, seed=3)
    n_bad = check_assignments_lazy(r["assignments"].cpu().numpy(), o["assignments"], x, o["centroids"], "fit of one iteration")
    if n_bad == 0:
        assert (r["counts"].cpu().numpy() == o["counts"]).all()
        check_values(host_matrix(r["centroids"]), o["centroids"], 1e-6, "centroids")
        check_values(host_matrix(r["gamma"]), o["gamma"], RTOL[dt], "gamma")
    np.testing.assert_allclose(r["inertia"].cpu().numpy(), o["inertia"], rtol=1e-4)


def test_captures_into_a_hip_graph_and_replays():
    N, D, K = 5000, 1001, 16
    x, cent, gamma, beta = _problem(3, N, D, K, "f32")
    xd = dev_matrix(x, "f32")
    c, g, b = (torch.from_numpy(a).cuda() for a in (cent, gamma, beta))
    ws = torch.empty(binding.cat_apply_workspace_bytes(N, D, K), dtype=torch.uint8, device="cuda")
    out = torch.empty_like(xd)

    def run():
        return cat_apply(xd, c, g, b, alpha=0.6, out=out, workspace=ws)

    ref_out, ref_a = (t.clone() for t in run())
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        o, a = run()
    for _ in range(3):
        o.zero_()
        a.zero_()
        ws.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(o, ref_out) and torch.equal(a, ref_a)
