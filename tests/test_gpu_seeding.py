"""GPU-vs-oracle parity of the D^2-weighted seeding (k-means++, Arthur and Vassilvitskii 2007).

The chosen rows are integers decided by a running sum in floating point; both sides sum in double, the oracle in
one sequential chain, the library in fixed groups.  The two agree unless a draw falls within rounding (about 1e-13
of the total) of a running sum, which the seeded cases here do not hit; every case therefore compares the row
numbers exactly, and the centroids bit for bit with the rows of the input."""
import numpy as np
import pytest
import torch

import oracle
from paper_2509_26277_amd import cat_fit, cat_init_kmeanspp, workloads
from paper_2509_26277_amd.binding import CatError

from parity_util import dev_matrix

pytestmark = pytest.mark.gpu


CASES = [
    # N, D, K, dtype
    (1000, 64, 8, "f32"),
    (4097, 1000, 16, "f32"),   # ragged last group of rows
    (777, 37, 5, "f32"),       # D not a multiple of 4: one channel per lane
    (3000, 256, 32, "bf16"),
    (515, 12, 3, "bf16"),      # 24-byte rows: narrow path
    (64, 8, 64, "f32"),        # every row becomes a centre
    (70000, 16, 4, "f32"),     # more partial sums than threads of the picking workgroup
    (300, 2048, 6, "bf16"),
    (5, 3, 1, "f32"),
]


@pytest.mark.parametrize("N,D,K,dt", CASES)
def test_rows_match_the_oracle(N, D, K, dt):
    rng = np.random.default_rng(N + 3 * D + K)
    centres = rng.standard_normal((max(K // 2, 1), D)) * 3
    x = (centres[rng.integers(0, len(centres), N)] + rng.standard_normal((N, D))).astype(np.float32)
    if dt == "bf16":
        x = workloads.round_to_bf16(x)
    for seed in (0, 12345):
        want = oracle.kmeanspp(x, K, seed=seed)
        cent, idx = cat_init_kmeanspp(dev_matrix(x, dt), K, seed=seed)
        got = idx.cpu().numpy()
        assert got.tolist() == want.tolist(), (seed, got, want)
        assert (cent.cpu().numpy() == x[want]).all()


def test_degenerate_rows():
    same = np.ones((130, 8), dtype=np.float32)
    want = oracle.kmeanspp(same, 5, seed=7)
    _, idx = cat_init_kmeanspp(dev_matrix(same, "f32"), 5, seed=7)
    assert idx.cpu().numpy().tolist() == want.tolist()
    two = np.zeros((200, 4), dtype=np.float32)
    two[100:] = 5.0
    for seed in range(4):
        want = oracle.kmeanspp(two, 4, seed=seed)
        _, idx = cat_init_kmeanspp(dev_matrix(two, "f32"), 4, seed=seed)
        assert idx.cpu().numpy().tolist() == want.tolist()


def test_seeds_a_fit_that_reaches_the_planted_partition():
    """on the planted mixture the seeding puts one centre in (almost) every component, and the fit started from it
    ends at an objective no worse than the fit started from uniformly drawn rows"""
    w = workloads.make("cfg1")
    x, y, K = w["lq"], w["fp"], w["K"]
    xd, yd = dev_matrix(x, "f32"), dev_matrix(y, "f32")
    cent, idx = cat_init_kmeanspp(xd, K, seed=3)
    assert idx.cpu().numpy().tolist() == oracle.kmeanspp(x, K, seed=3).tolist()
    r_pp = cat_fit(xd, yd, K, w["iters"], init_centroids=cent)
    r_uni = cat_fit(xd, yd, K, w["iters"], seed=3)
    j_pp, j_uni = float(r_pp["inertia"][-1]), float(r_uni["inertia"][-1])
    assert j_pp <= j_uni * (1 + 1e-6)
    # and the oracle, started from the same rows, ends in the same partition
    o = oracle.fit(x, y, K, w["iters"], init_centroids=x[idx.cpu().numpy()].astype(np.float64))
    assert (r_pp["assignments"].cpu().numpy() == o["assignments"]).all()


def test_full_logit_workload():
    """all of cfg2 (65,536 x 1000, K = 16)"""
    w = workloads.make("cfg2")
    want = oracle.kmeanspp(w["lq"], w["K"], seed=w["seed"])
    _, idx = cat_init_kmeanspp(dev_matrix(w["lq"], "f32"), w["K"], seed=w["seed"])
    assert idx.cpu().numpy().tolist() == want.tolist()
    assert len(set(want.tolist())) == w["K"]


def test_bad_arguments_are_refused():
    x = torch.zeros((10, 4), device="cuda")
    with pytest.raises(CatError):
        cat_init_kmeanspp(x, 11)
    with pytest.raises(CatError):
        cat_init_kmeanspp(x, 0)
    with pytest.raises(CatError):
        cat_init_kmeanspp(x, 2, workspace=torch.empty(256, dtype=torch.uint8, device="cuda")[:64])
