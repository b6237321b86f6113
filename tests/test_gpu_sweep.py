"""GPU-vs-oracle parity of the sweep over the blending coefficient (the alpha display of Sec. 3.1; the
ablation on alpha of Sec. 5): Top-1 position per row and alpha, Top-1 hits, squared error to FP.

Top-1 is an argmax decided in floating point.  The library decides it on fp32 values, the oracle on
doubles; rows whose two largest corrected entries are closer than MARGIN_TOL times the size of the
entries may differ, and then the library's choice must still be one of the near-largest entries.  Where
all arithmetic is exact (small integers) the comparison is bit for bit, ties included."""
import numpy as np
import pytest
import torch

import oracle
from paper_2509_26277_amd import cat_alpha_sweep, cat_top1, workloads
from paper_2509_26277_amd.binding import CatError

from parity_util import dev_matrix

pytestmark = pytest.mark.gpu

MARGIN_TOL = 4e-6   # a few fp32 roundings of the corrected value, relative to the largest entry size
SQ_RTOL = 2e-6      # per-lane fp32 partial sums of at most D / 64 squares, then doubles

ALPHAS10 = [0.1 * k for k in range(1, 11)]  # the grid of the paper's ablation figures


def _params(rng, K, D):
    return rng.uniform(0.4, 1.6, (K, D)).astype(np.float32), (rng.standard_normal((K, D)) * 0.7).astype(np.float32)


def _corrected(x, a, g, b, alpha, K):
    """test-side check values for the rows the tolerance exempts (double)"""
    x = x.astype(np.float64)
    inside = (a >= 0) & (a < K)
    ac = np.where(inside, a, 0)
    t = np.where(inside[:, None], x * (g.astype(np.float64)[ac] - 1.0) + b.astype(np.float64)[ac], 0.0)
    return x + alpha * t


def _check(x, a, g, b, alphas, K, res, ora, fp=None, labels=None):
    al32 = np.asarray(alphas, dtype=np.float32)
    N = x.shape[0]
    if res["top1"] is not None:
        got = res["top1"].cpu().numpy()
        assert got.shape == (N, len(alphas))
        for s, alpha in enumerate(al32):
            diff = np.flatnonzero(got[:, s] != ora["top1"][:, s])
            if diff.size == 0:
                continue
            c = _corrected(x[diff], a[diff], g, b, float(alpha), K)
            size = np.abs(c).max(axis=1)
            assert (ora["margin"][diff, s] <= MARGIN_TOL * size).all(), (
                f"alpha[{s}]: rows with a clear margin differ, e.g. row {diff[0]}")
            chosen = c[np.arange(diff.size), got[diff, s]]
            assert (chosen >= c.max(axis=1) - MARGIN_TOL * size).all()
    if labels is not None:
        hits = res["hits"].cpu().numpy()
        if res["top1"] is not None:  # the count is that of the library's own Top-1
            assert (hits == (res["top1"].cpu().numpy() == labels[:, None]).sum(axis=0)).all()
        for s in range(len(alphas)):
            c = _corrected(x, a, g, b, float(al32[s]), K)
            loose = int((ora["margin"][:, s] <= MARGIN_TOL * np.abs(c).max(axis=1)).sum())
            assert abs(int(hits[s]) - int(ora["hits"][s])) <= loose, (s, hits[s], ora["hits"][s], loose)
    if fp is not None:
        np.testing.assert_allclose(res["sq_err"].cpu().numpy(), ora["sq_err"], rtol=SQ_RTOL)
        m = res["moments"].cpu().numpy()
        al = al32.astype(np.float64)
        np.testing.assert_allclose(res["sq_err"].cpu().numpy(), m[0] + 2 * al * m[1] + al * al * m[2], rtol=1e-12)
        assert m[0] >= 0 and m[2] >= 0


CASES = [
    # N, D, K, dtype, alphas
    (1000, 64, 4, "f32", ALPHAS10),
    (777, 1000, 16, "f32", ALPHAS10),       # the paper's logit width: one whole double step and a ragged rest
    (500, 1001, 3, "f32", [0.0, 0.5, 1.0]),  # D not a multiple of 4: the one-entry path
    (300, 130, 5, "f32", [0.3] * 1),
    (1200, 256, 8, "bf16", [0.05 * k for k in range(16)]),  # the longest list
    (640, 512, 7, "f32", [1.0, 0.25]),      # exactly one double step, no rest
    (333, 1024, 2, "bf16", ALPHAS10),
    (257, 508, 9, "f32", [0.6, -0.2, 1.5, 0.9, 0.1, 0.7, 0.3, 0.2, 1.1, 0.0, 0.4, 0.8]),  # twelve values
    (64, 4, 2, "f32", [0.5, 1.0]),
    (50, 1, 1, "f32", [0.7]),
    (5000, 36, 6, "bf16", [0.2, 0.4, 0.6, 0.8]),
]


@pytest.mark.parametrize("N,D,K,dt,alphas", CASES)
def test_sweep_matches_the_oracle(N, D, K, dt, alphas):
    rng = np.random.default_rng(N * 7 + D)
    x = (rng.standard_normal((N, D)) * 2).astype(np.float32)
    y = (x * rng.uniform(0.6, 1.4, D).astype(np.float32) + rng.standard_normal((N, D)).astype(np.float32) * 0.5).astype(np.float32)
    if dt == "bf16":
        x, y = workloads.round_to_bf16(x), workloads.round_to_bf16(y)
    g, b = _params(rng, K, D)
    a = rng.integers(0, K, N).astype(np.int32)
    lab = rng.integers(0, D, N).astype(np.int32)
    lab[::3] = np.argmax(y, axis=1)[::3]
    al32 = np.asarray(alphas, dtype=np.float32)
    ora = oracle.alpha_sweep(x, a, g, b, al32.astype(np.float64), fp=y, labels=lab)
    res = cat_alpha_sweep(dev_matrix(x, dt), torch.from_numpy(a).cuda(), torch.from_numpy(g).cuda(), torch.from_numpy(b).cuda(),
                          alphas, fp=dev_matrix(y, dt), labels=torch.from_numpy(lab).cuda(), want_top1=True)
    _check(x, a, g, b, alphas, K, res, ora, fp=y, labels=lab)


def test_each_output_alone_gives_the_same_numbers():
    rng = np.random.default_rng(5)
    N, D, K = 900, 200, 5
    x = (rng.standard_normal((N, D)) * 2).astype(np.float32)
    y = (x + rng.standard_normal((N, D)).astype(np.float32)).astype(np.float32)
    g, b = _params(rng, K, D)
    a = rng.integers(0, K, N).astype(np.int32)
    lab = np.argmax(y, axis=1).astype(np.int32)
    xd, yd, ad, gd, bd, ld = (dev_matrix(x, "f32"), dev_matrix(y, "f32"), torch.from_numpy(a).cuda(), torch.from_numpy(g).cuda(),
                              torch.from_numpy(b).cuda(), torch.from_numpy(lab).cuda())
    al = [0.0, 0.4, 1.0]
    full = cat_alpha_sweep(xd, ad, gd, bd, al, fp=yd, labels=ld, want_top1=True)
    only_hits = cat_alpha_sweep(xd, ad, gd, bd, al, labels=ld)
    only_err = cat_alpha_sweep(xd, ad, gd, bd, al, fp=yd)
    only_top = cat_alpha_sweep(xd, ad, gd, bd, al, want_top1=True)
    assert only_hits["sq_err"] is None and only_hits["top1"] is None and only_err["hits"] is None
    assert torch.equal(only_hits["hits"], full["hits"])
    assert torch.equal(only_top["top1"], full["top1"])
    np.testing.assert_allclose(only_err["sq_err"].cpu().numpy(), full["sq_err"].cpu().numpy(), rtol=1e-12)
    ora = oracle.alpha_sweep(x, a, g, b, np.asarray(al, np.float32).astype(np.float64), fp=y, labels=lab)
    _check(x, a, g, b, al, K, full, ora, fp=y, labels=lab)
    # alpha = 0 counts the Top-1 agreement of the uncorrected rows
    assert int(full["hits"][0]) == int((np.argmax(x, axis=1) == lab).sum())


@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_exact_arithmetic_is_bit_for_bit_ties_included(dt):
    """small integers: every product and sum is exact in fp32 and in double, ties are real ties"""
    rng = np.random.default_rng(11)
    N, D, K = 2000, 24, 3
    x = rng.integers(-2, 3, (N, D)).astype(np.float32)
    y = rng.integers(-2, 3, (N, D)).astype(np.float32)
    g = rng.integers(0, 3, (K, D)).astype(np.float32)
    b = rng.integers(-1, 2, (K, D)).astype(np.float32)
    a = rng.integers(-1, K + 1, N).astype(np.int32)  # -1 and K: rows without a cluster
    lab = rng.integers(-1, D + 1, N).astype(np.int32)  # labels outside [0, D) never match
    al = [0.0, 0.5, 1.0, 2.0]
    ora = oracle.alpha_sweep(x, a, g, b, al, fp=y, labels=lab)
    assert (ora["margin"] == 0).mean() > 0.2  # the case is about ties
    res = cat_alpha_sweep(dev_matrix(x, dt), torch.from_numpy(a).cuda(), torch.from_numpy(g).cuda(), torch.from_numpy(b).cuda(), al,
                          fp=dev_matrix(y, dt), labels=torch.from_numpy(lab).cuda(), want_top1=True)
    assert (res["top1"].cpu().numpy() == ora["top1"]).all()
    assert (res["hits"].cpu().numpy() == ora["hits"]).all()
    assert (res["sq_err"].cpu().numpy() == ora["sq_err"]).all()


def test_rows_that_do_not_start_on_a_16_byte_boundary():
    rng = np.random.default_rng(13)
    N, D, K = 300, 64, 4
    x = (rng.standard_normal((N, D)) * 2).astype(np.float32)
    y = (x + rng.standard_normal((N, D)).astype(np.float32)).astype(np.float32)
    g, b = _params(rng, K, D)
    a = rng.integers(0, K, N).astype(np.int32)
    lab = np.argmax(y, axis=1).astype(np.int32)
    flat = torch.empty(N * D + 1, dtype=torch.float32, device="cuda")
    xd = flat[1:].view(N, D)
    xd.copy_(torch.from_numpy(x))
    assert xd.data_ptr() % 16 != 0
    res = cat_alpha_sweep(xd, torch.from_numpy(a).cuda(), torch.from_numpy(g).cuda(), torch.from_numpy(b).cuda(), ALPHAS10,
                          fp=dev_matrix(y, "f32"), labels=torch.from_numpy(lab).cuda(), want_top1=True)
    ora = oracle.alpha_sweep(x, a, g, b, np.asarray(ALPHAS10, np.float32).astype(np.float64), fp=y, labels=lab)
    _check(x, a, g, b, ALPHAS10, K, res, ora, fp=y, labels=lab)


def test_fitted_parameters_put_the_best_alpha_at_one():
    """gamma, beta from the oracle's least-squares fit on the same rows: the squared error is smallest at
    alpha = 1 (the residual is orthogonal to the correction), which the three sums must reproduce"""
    w = workloads.make("cfg1", n_rows=3000)
    x, y, K = w["lq"], w["fp"], w["K"]
    a = w["labels"].astype(np.int32)
    g64, b64, _ = oracle.affine(x, y, a, K)
    g, b = g64.astype(np.float32), b64.astype(np.float32)
    res = cat_alpha_sweep(dev_matrix(x, "f32"), torch.from_numpy(a).cuda(), torch.from_numpy(g).cuda(), torch.from_numpy(b).cuda(),
                          [0.0, 0.5, 1.0, 1.5], fp=dev_matrix(y, "f32"))
    m = res["moments"].cpu().numpy()
    assert abs(-m[1] / m[2] - 1.0) < 1e-4
    sq = res["sq_err"].cpu().numpy()
    assert sq[2] < sq[1] < sq[0] and sq[2] < sq[3]
    np.testing.assert_allclose(sq, oracle.alpha_sweep(x, a, g, b, [0.0, 0.5, 1.0, 1.5], fp=y)["sq_err"], rtol=SQ_RTOL)


@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("N,D", [(1000, 1000), (513, 37), (64, 1), (300, 516)])
def test_top1_of_rows(N, D, dt):
    rng = np.random.default_rng(N + D)
    x = np.round(rng.standard_normal((N, D)) * 4).astype(np.float32) / 2  # halves: plenty of exact ties
    none = np.full(N, -1, dtype=np.int32)
    one = np.ones((1, D), dtype=np.float32)
    want = oracle.alpha_sweep(x, none, one, 0 * one, [0.0])["top1"][:, 0]
    got = cat_top1(dev_matrix(x, dt)).cpu().numpy()
    assert (got == want).all()


def test_bad_arguments_are_refused():
    N, D, K = 16, 8, 2
    x = torch.zeros((N, D), device="cuda")
    a = torch.zeros((N,), dtype=torch.int32, device="cuda")
    g = torch.ones((K, D), device="cuda")
    lab = torch.zeros((N,), dtype=torch.int32, device="cuda")
    with pytest.raises(CatError):
        cat_alpha_sweep(x, a, g, g, [], labels=lab)
    with pytest.raises(CatError):
        cat_alpha_sweep(x, a, g, g, [0.1] * 17, labels=lab)
    with pytest.raises(CatError):
        cat_alpha_sweep(x, a, g, g, [float("nan")], labels=lab)
    with pytest.raises(CatError):
        cat_alpha_sweep(x, a, g, g, [0.5])  # nothing asked for
    small = torch.empty(64, dtype=torch.uint8, device="cuda")
    with pytest.raises(CatError):
        cat_alpha_sweep(x, a, g, g, [0.5], labels=lab, workspace=small)


def test_full_logit_workload_in_the_benchmark_configuration():
    """all of cfg2 (65,536 x 1000, K = 16) with the ten-value grid: every row against the oracle"""
    w = workloads.make("cfg2")
    x, y, K = w["lq"], w["fp"], w["K"]
    a = w["labels"].astype(np.int32)
    g64, b64, _ = oracle.affine(x, y, a, K)
    g, b = g64.astype(np.float32), b64.astype(np.float32)
    xd, yd = dev_matrix(x, "f32"), dev_matrix(y, "f32")
    lab_d = cat_top1(yd)
    lab = np.argmax(y, axis=1).astype(np.int32)
    assert (lab_d.cpu().numpy() == lab).all()
    al32 = np.asarray(ALPHAS10, dtype=np.float32)
    ora = oracle.alpha_sweep(x, a, g, b, al32.astype(np.float64), fp=y, labels=lab)
    res = cat_alpha_sweep(xd, torch.from_numpy(a).cuda(), torch.from_numpy(g).cuda(), torch.from_numpy(b).cuda(), ALPHAS10,
                          fp=yd, labels=lab_d, want_top1=True)
    _check(x, a, g, b, ALPHAS10, K, res, ora, fp=y, labels=lab)
    # the correction helps: agreement with the FP Top-1 rises from alpha = 0.1 to alpha = 1
    hits = res["hits"].cpu().numpy()
    assert hits[-1] > hits[0]
