"""The row-tile inference kernel (the fused cat_apply kernel that reads every row once) against the oracle.

Every case forces that kernel (cat_debug_apply_kernel(2)), so a shape it has no instance for fails loudly instead of
passing on the other kernel; the result is also compared with the tile kernel's, which must agree bit for bit in the
corrected rows wherever the two assign the same cluster.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2509_26277_amd import binding, cat_apply, workloads

from parity_util import RTOL, check_assignments, check_values, dev_matrix, host_matrix

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _automatic_after():
    yield
    binding.debug_apply_kernel(0)


def _mixture(N, D, K, seed, spread=1.0, dtype="f32"):
    rng = np.random.default_rng(seed)
    cent = (spread * rng.standard_normal((K, D))).astype(np.float32)
    gamma = rng.uniform(0.8, 1.2, (K, D)).astype(np.float32)
    beta = (0.3 * rng.standard_normal((K, D))).astype(np.float32)
    lq = (cent[rng.integers(0, K, N)] + rng.standard_normal((N, D))).astype(np.float32)
    if dtype == "bf16":
        lq = workloads.round_to_bf16(lq)
    return lq, cent, gamma, beta


def _run(lq, cent, gamma, beta, dtype, alpha, which):
    binding.debug_apply_kernel(which)
    out, a = cat_apply(dev_matrix(lq, dtype), *(torch.from_numpy(x).cuda() for x in (cent, gamma, beta)), alpha=alpha)
    torch.cuda.synchronize()
    return out, a.cpu().numpy()


# (N, D, K, spread): shapes of the inference workload (K = 128, D = 512), of the logit workload (K = 16, D = 1000), of
# the feature-map workload (K = 32, D = 256); several tiles and a ragged last one; K off the 16-cluster tile; rows
# shorter than one vector round; overlapping clusters (spread 0.05: nearly every row goes through the exact re-rank)
SHAPES = [(16 * 700 + 5, 512, 128, 1.0), (4099, 1000, 16, 1.0), (9001, 256, 32, 1.0), (3000, 512, 100, 0.05),
          (1, 512, 1, 1.0), (130, 512, 128, 1.0), (15, 64, 3, 1.0), (37, 260, 19, 0.3), (2500, 8, 5, 1.0), (5003, 1000, 9, 0.05),
          (4000, 384, 64, 0.2), (3333, 128, 128, 0.5), (2048, 768, 24, 1.0)]


@pytest.mark.parametrize("alpha", [1.0, 0.6])
@pytest.mark.parametrize("N,D,K,spread", SHAPES)
def test_row_tile_kernel_against_the_oracle(N, D, K, spread, alpha):
    lq, cent, gamma, beta = _mixture(N, D, K, seed=N + D + K, spread=spread)
    out, a = _run(lq, cent, gamma, beta, "f32", alpha, which=2)
    o_out, o_a = oracle.apply(lq, cent, gamma, beta, alpha)
    _, d1, d2 = oracle.assign(lq, cent.astype(np.float64), want_distances=True)
    check_assignments(a, o_a, d1, d2, "row-tile kernel, assignments")
    same = a == o_a
    check_values(host_matrix(out)[same], o_out[same], RTOL["f32"], "row-tile kernel, corrected")
    out1, a1 = _run(lq, cent, gamma, beta, "f32", alpha, which=1)
    both = a == a1
    assert both.mean() > 0.999 or spread < 0.1
    assert torch.equal(out[torch.from_numpy(both).cuda()], out1[torch.from_numpy(both).cuda()])


@pytest.mark.parametrize("N,D,K,spread", [(5003, 512, 16, 1.0), (3001, 1024, 30, 0.3), (2000, 256, 64, 0.05), (777, 8, 3, 1.0)])
def test_row_tile_kernel_on_bf16_rows(N, D, K, spread):
    lq, cent, gamma, beta = _mixture(N, D, K, seed=N + D, spread=spread, dtype="bf16")
    out, a = _run(lq, cent, gamma, beta, "bf16", 0.8, which=2)
    o_out, o_a = oracle.apply(lq, cent, gamma, beta, 0.8)
    _, d1, d2 = oracle.assign(lq, cent.astype(np.float64), want_distances=True)
    check_assignments(a, o_a, d1, d2, "row-tile kernel, bf16 rows, assignments")
    same = a == o_a
    check_values(host_matrix(out)[same], o_out[same], RTOL["bf16"], "row-tile kernel, bf16 rows, corrected")
    out1, a1 = _run(lq, cent, gamma, beta, "bf16", 0.8, which=1)
    both = torch.from_numpy(a == a1).cuda()
    assert torch.equal(out[both].view(torch.int16), out1[both].view(torch.int16))


def test_exact_ties_go_to_the_lowest_index():
    """Duplicated centroids and rows at exact midpoints, in half-integers so that all arithmetic is exact."""
    rng = np.random.default_rng(7)
    D = 64
    base = np.round(rng.standard_normal((3, D)) * 4) / 2
    cent = np.stack([base[0], base[1], base[1], base[2], base[0]]).astype(np.float32)
    rows = [base[1], base[0], (base[1] + base[2]) / 2, (base[0] + base[2]) / 2]
    rows += [base[i % 3] + np.round(rng.standard_normal(D) * 2) / 4 for i in range(200)]
    lq = np.stack(rows).astype(np.float32)
    gamma = np.ones_like(cent)
    beta = np.arange(5, dtype=np.float32)[:, None] * np.ones((1, D), np.float32)  # beta = cluster index
    o_out, o_a = oracle.apply(lq, cent, gamma, beta, 1.0)
    assert o_a[:4].tolist() == [1, 0, 1, 0]
    out, a = _run(lq, cent, gamma, beta, "f32", 1.0, which=2)
    assert a.tolist() == o_a.tolist()
    assert (host_matrix(out) == o_out).all()


def test_forcing_it_on_a_shape_without_an_instance_is_an_error():
    lq, cent, gamma, beta = _mixture(400, 8, 300, seed=1)  # more than 256 clusters
    with pytest.raises(binding.CatError) as e:
        _run(lq, cent, gamma, beta, "f32", 1.0, which=2)
    assert e.value.status == 2
