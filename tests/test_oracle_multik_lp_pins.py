"""Pins of the oracle's fits for several cluster counts (a plain loop over the pinned single fit) and of its
low-precision deployment (bfloat16 rounding from the definition of the format, then the pinned inference)."""
import numpy as np
import torch

import oracle


def _mixture(seed, N, D, comps, spread=4.0):
    rng = np.random.default_rng(seed)
    centres = rng.standard_normal((comps, D)) * spread
    x = (centres[rng.integers(0, comps, N)] + rng.standard_normal((N, D))).astype(np.float32)
    y = (0.9 * x + 0.3 + 0.05 * rng.standard_normal((N, D))).astype(np.float32)
    return x, y


def test_multi_k_is_the_single_fit_per_cluster_count():
    x, y = _mixture(3, 400, 6, 5)
    Ks = [1, 8, 16, 24, 3]
    runs = oracle.fit_multi_k(x, y, Ks, 4, seed=9)
    assert len(runs) == len(Ks)
    for K, r in zip(Ks, runs):
        one = oracle.fit(x, y, K, 4, seed=9)
        assert r["centroids"].shape == (K, 6)
        for key in ("centroids", "gamma", "beta", "assignments", "counts", "inertia"):
            assert (np.asarray(r[key]) == np.asarray(one[key])).all(), (K, key)
    # K = 1: the plain per-channel least-squares line (the paper's "plain affine" baseline)
    g, b = runs[0]["gamma"][0], runs[0]["beta"][0]
    for j in range(6):
        slope, icpt = np.polyfit(x[:, j].astype(np.float64), y[:, j].astype(np.float64), 1)
        assert abs(g[j] - slope) < 1e-9 and abs(b[j] - icpt) < 1e-9


def test_more_clusters_never_raise_the_optimum_on_nested_inits():
    # a sanity property of the grid: with the seeded rows of K as a prefix of those of K' > K (same seed, same
    # walk), the starting objective of K' is at most that of K
    x, y = _mixture(5, 300, 4, 6)
    runs = oracle.fit_multi_k(x, y, [2, 4, 8], 0, seed=1)
    idx = [oracle.init_indices(300, K, 1) for K in (2, 4, 8)]
    assert list(idx[1][:2]) == list(idx[0]) and list(idx[2][:4]) == list(idx[1])
    assert runs[0]["inertia"][0] >= runs[1]["inertia"][0] >= runs[2]["inertia"][0]


def test_bf16_rounding_by_hand():
    # 1 + 2^-8 lies halfway between 1 and 1 + 2^-7: ties go to the even significand (1); 1 + 3 * 2^-8 is halfway
    # between 1 + 2^-7 and 1 + 2^-6 and goes to the even one, 1 + 2^-6
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, -(1.0 + 2.0 ** -8), 0.0, 0.1,
                  3.0e-5, 255.0, 257.0, 65535.0])
    want = np.array([1.0, 1.0, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7, -1.0, 0.0, 0.10009765625, 252 * 2.0 ** -23,  # 3.0e-5 = 251.66 * 2^-23
                     255.0, 256.0, 65536.0])
    assert (oracle.to_bf16(x) == want).all()


def test_bf16_rounding_against_the_library_conversion():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(20000) * 10.0 ** rng.integers(-6, 7, 20000),
                        (np.arange(-512, 512) + 0.5) * 2.0 ** -8 + 1.0]).astype(np.float32)  # includes exact ties
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    assert (oracle.to_bf16(x.astype(np.float64)) == want).all()
    q = oracle.to_bf16(x.astype(np.float64))
    assert (oracle.to_bf16(q) == q).all()  # idempotent
    assert (np.abs(q - x) <= np.abs(x) * 2.0 ** -8).all()  # half a unit in the last of 8 bits, relative to x


def test_low_precision_inference():
    x, y = _mixture(11, 500, 7, 4)
    r = oracle.fit(x, y, 4, 5, seed=2)
    out, a, (cq, gq, bq) = oracle.apply_lp(x, r["centroids"], r["gamma"], r["beta"], alpha=0.6)
    # the parameters it used are bfloat16 values, and the result is the pinned inference on them, rounded
    for p, p0 in ((cq, r["centroids"]), (gq, r["gamma"]), (bq, r["beta"])):
        assert (torch.from_numpy(p).to(torch.bfloat16).to(torch.float64).numpy() == p).all()
        assert (np.abs(p - p0) <= np.abs(p0) * 2.0 ** -8).all()
    ref, a_ref = oracle.apply(x, cq, gq, bq, 0.6)
    assert (a == a_ref).all()
    assert (out == oracle.to_bf16(ref)).all()
    out32, _, _ = oracle.apply_lp(x, r["centroids"], r["gamma"], r["beta"], alpha=0.6, bf16_out=False)
    assert (out32 == ref).all()
    # parameters that are bfloat16 values already: identical to the plain inference, up to the output rounding
    o2, a2, _ = oracle.apply_lp(x, cq, gq, bq, alpha=1.0, bf16_out=False)
    o3, a3 = oracle.apply(x, cq, gq, bq, 1.0)
    assert (o2 == o3).all() and (a2 == a3).all()
    # low precision costs little: the corrected rows stay within a few bfloat16 steps of the full-precision ones
    full, _ = oracle.apply(x, r["centroids"], r["gamma"], r["beta"], 0.6)
    same = a == oracle.assign(x, r["centroids"])
    assert same.mean() > 0.99
    assert np.abs(out - full)[same].max() <= 0.05 * np.abs(full).max()
