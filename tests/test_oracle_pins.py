"""Pins for the CPU oracle: everything here checks ``oracle/`` against something
other than itself -- published vectors, a hand example, library routines
(numpy / scipy / scikit-learn), closed forms, invariants and brute force.

CPU only.  The GPU library is not touched.
"""
import itertools
import os

import numpy as np
import pytest
from scipy.cluster.vq import kmeans2
from scipy.spatial.distance import cdist

import oracle
from paper_2509_26277_amd import workloads

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _read_golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            out[key] = vals
    return out


# ---------------------------------------------------------------------------
# seeded initialisation
# ---------------------------------------------------------------------------
def test_splitmix64_published_vectors():
    with open(os.path.join(GOLDEN, "splitmix64_vectors.txt")) as f:
        rows = [l.split() for l in f if l.strip() and not l.startswith("#")]
    assert len(rows) == 2
    for seed, *outs in rows:
        got = [oracle.splitmix64(int(seed), t) for t in range(len(outs))]
        assert got == [int(v) for v in outs]


def test_init_indices_distinct_in_range_and_follow_the_stream():
    N, K, seed = 37, 30, 99  # K close to N forces rejections
    idx = oracle.init_indices(N, K, seed)
    assert len(set(idx.tolist())) == K and idx.min() >= 0 and idx.max() < N
    # replay the documented rule with python integers
    want, t = [], 0
    while len(want) < K:
        z = (seed + (t + 1) * 0x9E3779B97F4A7C15) % 2**64
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) % 2**64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) % 2**64
        z ^= z >> 31
        t += 1
        if z % N not in want:
            want.append(z % N)
    assert idx.tolist() == want
    assert t > K  # the case really exercised a rejection


# ---------------------------------------------------------------------------
# the hand example (exact in binary)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("iters", [1, 2, 5])
def test_hand_example_exact(iters):
    g = _read_golden("hand_example.txt")
    lq = np.array(g["lq"], dtype=np.float32)[:, None]
    fp = np.array(g["fp"], dtype=np.float32)[:, None]
    init = lq[[int(r) for r in g["init_rows"]]].astype(np.float64)
    r = oracle.fit(lq, fp, K=2, iters=iters, init_centroids=init)
    assert r["assignments"].tolist() == [int(v) for v in g["assignments"]]
    assert r["centroids"][:, 0].tolist() == [float(v) for v in g["centroids"]]
    assert r["gamma"][:, 0].tolist() == [float(v) for v in g["gamma"]]
    assert r["beta"][:, 0].tolist() == [float(v) for v in g["beta"]]
    assert r["counts"].tolist() == [2, 2]
    assert r["inertia"][0] == float(g["inertia_first"][0])
    assert all(v == float(g["inertia_later"][0]) for v in r["inertia"][1:])
    for alpha in ("1", "0.5", "0"):
        out, a = oracle.apply(lq, r["centroids"], r["gamma"], r["beta"], alpha=float(alpha))
        assert out[:, 0].tolist() == [float(v) for v in g["corrected_alpha_" + alpha]]
        assert a.tolist() == r["assignments"].tolist()


# ---------------------------------------------------------------------------
# K = 1: plain affine transformation == per-channel ordinary least squares
# ---------------------------------------------------------------------------
def test_k1_is_per_channel_least_squares():
    rng = np.random.default_rng(7)
    N, D = 500, 6
    lq = rng.standard_normal((N, D)).astype(np.float32) * 3 + 1.5
    fp = (0.7 * lq + 0.3 + rng.standard_normal((N, D)) * 0.4).astype(np.float32)
    r = oracle.fit(lq, fp, K=1, iters=3, seed=5)
    for j in range(D):
        slope, icpt = np.polyfit(lq[:, j].astype(np.float64), fp[:, j].astype(np.float64), 1)
        assert r["gamma"][0, j] == pytest.approx(slope, rel=1e-10)
        assert r["beta"][0, j] == pytest.approx(icpt, rel=1e-9, abs=1e-12)
    np.testing.assert_allclose(r["centroids"][0], lq.astype(np.float64).mean(axis=0), rtol=1e-13)
    assert r["assignments"].max() == 0 and r["counts"].tolist() == [N]
    # objective of K = 1 after the first update = N * total population variance
    assert r["inertia"][-1] == pytest.approx(N * lq.astype(np.float64).var(axis=0).sum(), rel=1e-12)


# ---------------------------------------------------------------------------
# affine fit: normal equations, mean matching, edge cases
# ---------------------------------------------------------------------------
def _random_problem(seed, N=400, D=5, K=3):
    rng = np.random.default_rng(seed)
    lq = rng.standard_normal((N, D)).astype(np.float32) * 2
    fp = (rng.uniform(0.5, 1.5, D) * lq + rng.standard_normal((N, D))).astype(np.float32)
    a = rng.integers(0, K, N).astype(np.int32)
    return lq, fp, a


def test_affine_normal_equations_and_mean_matching():
    lq, fp, a = _random_problem(11)
    K = 3
    gamma, beta, counts = oracle.affine(lq, fp, a, K)
    assert counts.tolist() == np.bincount(a, minlength=K).tolist()
    x, y = lq.astype(np.float64), fp.astype(np.float64)
    for k in range(K):
        m = a == k
        res = y[m] - gamma[k] * x[m] - beta[k]
        assert np.abs(res.sum(axis=0)).max() < 1e-9          # sum r = 0
        assert np.abs((res * x[m]).sum(axis=0)).max() < 1e-8  # sum r x = 0
        # library check of the same numbers
        c = np.array([np.cov(x[m][:, j], y[m][:, j], bias=True)[0, 1] for j in range(x.shape[1])])
        np.testing.assert_allclose(gamma[k], c / x[m].var(axis=0), rtol=1e-11)
        np.testing.assert_allclose(beta[k], y[m].mean(axis=0) - gamma[k] * x[m].mean(axis=0), rtol=1e-11, atol=1e-13)


def test_affine_population_normalisation_shows_at_the_variance_floor():
    # n = 2, x = +-d with d^2 = 0.75e-8: population variance 0.75e-8 is below the
    # 1e-8 floor, the n-1 variance 1.5e-8 would not be.
    d = np.float32(np.sqrt(0.75e-8))
    lq = np.array([[-d], [d]], dtype=np.float32)
    fp = np.array([[-1.0], [1.0]], dtype=np.float32)
    gamma, beta, _ = oracle.affine(lq, fp, np.zeros(2, np.int32), 1)
    assert gamma[0, 0] == pytest.approx(float(d) / 1e-8, rel=1e-12)  # cov = d, var floored
    assert beta[0, 0] == pytest.approx(0.0, abs=1e-12)


def test_affine_constant_channel_single_row_and_empty_cluster():
    lq = np.array([[1.0, 5.0], [1.0, 7.0], [1.0, 9.0], [4.0, 4.0]], dtype=np.float32)
    fp = np.array([[2.0, 1.0], [3.0, 2.0], [7.0, 3.0], [8.0, 8.0]], dtype=np.float32)
    a = np.array([0, 0, 0, 2], dtype=np.int32)  # cluster 1 empty, cluster 2 one row
    gamma, beta, counts = oracle.affine(lq, fp, a, 3)
    assert counts.tolist() == [3, 0, 1]
    assert gamma[0, 0] == 0.0 and beta[0, 0] == 4.0          # constant LQ channel: gamma 0, beta = mean FP
    assert gamma[0, 1] == pytest.approx(0.5) and beta[0, 1] == pytest.approx(2.0 - 0.5 * 7.0)
    assert gamma[1].tolist() == [1.0, 1.0] and beta[1].tolist() == [0.0, 0.0]  # empty: identity
    assert gamma[2].tolist() == [0.0, 0.0] and beta[2].tolist() == [8.0, 8.0]  # one row


def test_planted_recovery_attenuated_inverse():
    # LQ = g FP + b + noise, CAT regresses FP on LQ: slope g s_F^2/(g^2 s_F^2 + s_n^2)
    w = workloads.planted_mixture(20000, 16, 4, seed=3)
    K = 4
    init = np.stack([w["lq"][np.flatnonzero(w["labels"] == k)[0]] for k in range(K)]).astype(np.float64)
    r = oracle.fit(w["lq"], w["fp"], K=K, iters=8, init_centroids=init)
    assert (r["assignments"] == w["labels"]).mean() > 0.999
    g, b, mu = w["g"].astype(np.float64), w["b"].astype(np.float64), w["mu"].astype(np.float64)
    sn2 = w["noise_std"] ** 2
    slope = g / (g * g + sn2)
    icpt = mu - slope * (g * mu + b)
    n_k = np.bincount(w["labels"], minlength=K)[:, None]
    se = 6.0 * (w["noise_std"] / g**2) / np.sqrt(n_k) + 1e-3
    assert (np.abs(r["gamma"] - slope) < se).all()
    assert (np.abs(r["beta"] - icpt) < se * (np.abs(g * mu + b) + 1.0)).all()


# ---------------------------------------------------------------------------
# assignment: library brute force, ties
# ---------------------------------------------------------------------------
def test_assign_matches_library_brute_force():
    rng = np.random.default_rng(2)
    N, D, K = 333, 7, 5  # K != D catches a transposed centroid index
    lq = rng.standard_normal((N, D)).astype(np.float32)
    cent = rng.standard_normal((K, D))
    a, d1, d2 = oracle.assign(lq, cent, want_distances=True)
    ref = cdist(lq.astype(np.float64), cent, "sqeuclidean")
    assert (a == ref.argmin(axis=1)).all()
    part = np.sort(ref, axis=1)
    np.testing.assert_allclose(d1, part[:, 0], rtol=1e-12)
    np.testing.assert_allclose(d2, part[:, 1], rtol=1e-12)
    np.testing.assert_allclose(oracle.distances(lq, cent), ref, rtol=1e-12)


def test_assign_ties_go_to_lowest_index():
    lq = np.array([[1.0, 1.0], [3.0, 3.0], [0.5, 0.5]], dtype=np.float32)
    cent = np.array([[4.0, 4.0], [0.0, 0.0], [0.0, 0.0], [2.0, 2.0], [4.0, 4.0]])
    a, d1, d2 = oracle.assign(lq, cent, want_distances=True)
    # row 0: midpoint of centroid 1/2 (duplicates) and 3 -> exact 3-way tie at 2.0 -> index 1
    # row 1: midpoint of 0/4 (duplicates) and 3 -> index 0
    assert a.tolist() == [1, 0, 1]
    assert d1.tolist() == [2.0, 2.0, 0.5] and d2.tolist() == [2.0, 2.0, 0.5]
    a1, _, d2_1 = oracle.assign(lq, cent[:1], want_distances=True)
    assert a1.tolist() == [0, 0, 0] and np.isinf(d2_1).all()


# ---------------------------------------------------------------------------
# Lloyd: library k-means, monotone objective, fixed point, exhaustive optimum
# ---------------------------------------------------------------------------
def test_lloyd_matches_scipy_kmeans2_iteration_by_iteration():
    w = workloads.planted_mixture(600, 5, 3, seed=21)
    lq = w["lq"]
    init = lq[[5, 17, 400]].astype(np.float64)
    for iters in (1, 2, 3, 6):
        r = oracle.fit(lq, w["fp"], K=3, iters=iters, init_centroids=init)
        cb, _ = kmeans2(lq.astype(np.float64), init.copy(), iter=iters, minit="matrix")
        np.testing.assert_allclose(r["centroids"], cb, rtol=1e-12, atol=1e-12)
        # returned assignments are those of the returned centroids
        assert (r["assignments"] == cdist(lq.astype(np.float64), cb, "sqeuclidean").argmin(axis=1)).all()


def test_lloyd_matches_sklearn_fixed_point():
    from sklearn.cluster import KMeans
    w = workloads.planted_mixture(900, 6, 4, seed=8)
    lq = w["lq"].astype(np.float64)
    init = lq[[0, 1, 2, 3]]
    r = oracle.fit(w["lq"], w["fp"], K=4, iters=60, init_centroids=init)
    km = KMeans(n_clusters=4, init=init, n_init=1, max_iter=300, tol=0.0, algorithm="lloyd").fit(lq)
    np.testing.assert_allclose(r["centroids"], km.cluster_centers_, rtol=1e-9, atol=1e-9)
    assert (r["assignments"] == km.labels_).all()
    assert r["inertia"][-1] == pytest.approx(km.inertia_, rel=1e-10)


def test_objective_is_non_increasing_and_reaches_a_fixed_point():
    w = workloads.logit_mixture(1500, 24, 5, seed=4)
    r = oracle.fit(w["lq"], w["fp"], K=5, iters=40, seed=12)
    J = r["inertia"]
    assert (np.diff(J) <= 1e-9 * J[:-1]).all() and J[-1] < J[0]
    # fixed point: nearest own centroid, centroid = mean of members
    a = oracle.assign(w["lq"], r["centroids"])
    assert (a == r["assignments"]).all()
    c2, n = oracle.update(w["lq"], a, r["centroids"])
    np.testing.assert_allclose(c2, r["centroids"], rtol=1e-12, atol=1e-12)
    assert n.sum() == 1500 and (n == r["counts"]).all()
    # inertia is the sum of direct-form squared distances
    d = cdist(w["lq"].astype(np.float64), r["centroids"], "sqeuclidean")
    assert J[-1] == pytest.approx(d.min(axis=1).sum(), rel=1e-12)


def test_empty_cluster_keeps_its_centroid_and_gets_identity_affine():
    w = workloads.planted_mixture(300, 4, 2, seed=5)
    lq = w["lq"]
    # (a) duplicate initial centroids: the later index never wins the tie, so it is empty
    #     in the first pass, keeps its place in the update, and (iters = 0) gets gamma 1, beta 0
    init = np.stack([lq[0], lq[0], lq[7]]).astype(np.float64)
    r0 = oracle.fit(lq, w["fp"], K=3, iters=0, init_centroids=init)
    assert r0["counts"][1] == 0 and (r0["assignments"] != 1).all()
    assert (r0["gamma"][1] == 1.0).all() and (r0["beta"][1] == 0.0).all()
    a = oracle.assign(lq, init)
    c1, n1 = oracle.update(lq, a, init)
    assert n1[1] == 0 and (c1[1] == init[1]).all() and not (c1[0] == init[0]).all()
    # (b) a centroid far from all data stays empty, and stays put, through every iteration
    far = np.stack([lq[0], np.full(4, 1e3), lq[7]]).astype(np.float64)
    r = oracle.fit(lq, w["fp"], K=3, iters=4, init_centroids=far)
    assert r["counts"][1] == 0 and (r["assignments"] != 1).all()
    assert (r["centroids"][1] == far[1]).all()
    assert (r["gamma"][1] == 1.0).all() and (r["beta"][1] == 0.0).all()
    assert (np.diff(r["inertia"]) <= 0).all()


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_tiny_inputs_against_exhaustive_optimum(seed):
    rng = np.random.default_rng(seed)
    N, D, K = 8, 2, 3
    centres = np.array([[0.0, 0.0], [20.0, 0.0], [0.0, 20.0]])
    lab = np.array([0, 0, 0, 1, 1, 1, 2, 2])
    lq = (centres[lab] + rng.standard_normal((N, D))).astype(np.float32)
    x = lq.astype(np.float64)
    best = np.inf
    for labeling in itertools.product(range(K), repeat=N):
        l = np.array(labeling)
        J = 0.0
        for k in range(K):
            if (l == k).any():
                J += ((x[l == k] - x[l == k].mean(axis=0)) ** 2).sum()
        best = min(best, J)
    init = x[[0, 3, 6]]
    r = oracle.fit(lq, lq, K=K, iters=10, init_centroids=init)
    assert r["inertia"][-1] == pytest.approx(best, rel=1e-12)  # well separated: Lloyd finds the optimum
    r2 = oracle.fit(lq, lq, K=K, iters=10, init_centroids=x[[0, 1, 2]])  # poor init: never below it
    assert r2["inertia"][-1] >= best * (1 - 1e-12)


# ---------------------------------------------------------------------------
# whole fit: invariances
# ---------------------------------------------------------------------------
def test_invariances_translation_fp_scaling_row_permutation():
    w = workloads.planted_mixture(800, 8, 3, seed=9)
    # keep every number exactly representable after the shift: snap to a coarse binary grid
    lq = (np.round(w["lq"] * 64) / 64).astype(np.float32)
    fp = (np.round(w["fp"] * 64) / 64).astype(np.float32)
    init = lq[[3, 30, 300]].astype(np.float64)
    base = oracle.fit(lq, fp, K=3, iters=7, init_centroids=init)

    t = np.arange(8, dtype=np.float32) * np.float32(0.5) - np.float32(1.0)
    sh = oracle.fit(lq + t, fp, K=3, iters=7, init_centroids=init + t)
    assert (sh["assignments"] == base["assignments"]).all()
    np.testing.assert_allclose(sh["centroids"], base["centroids"] + t, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(sh["gamma"], base["gamma"], rtol=1e-9)
    np.testing.assert_allclose(sh["beta"], base["beta"] - base["gamma"] * t, rtol=1e-9, atol=1e-9)

    s = np.array([2.0, 0.5, 4.0, 1.0, 8.0, 0.25, 1.0, 2.0], dtype=np.float32)
    sc = oracle.fit(lq, fp * s, K=3, iters=7, init_centroids=init)
    np.testing.assert_allclose(sc["gamma"], base["gamma"] * s, rtol=1e-12)
    np.testing.assert_allclose(sc["beta"], base["beta"] * s, rtol=1e-12, atol=1e-12)

    perm = np.random.default_rng(0).permutation(800)
    pm = oracle.fit(lq[perm], fp[perm], K=3, iters=7, init_centroids=init)
    assert (pm["assignments"] == base["assignments"][perm]).all()
    np.testing.assert_allclose(pm["centroids"], base["centroids"], rtol=1e-12)
    np.testing.assert_allclose(pm["gamma"], base["gamma"], rtol=1e-9)


# ---------------------------------------------------------------------------
# fit <-> apply
# ---------------------------------------------------------------------------
def test_apply_reproduces_fit_partition_and_alpha_semantics():
    w = workloads.relu_feature_map(2000, 12, 4, seed=6)
    r = oracle.fit(w["lq"], w["fp"], K=4, iters=6, seed=3)
    out1, a = oracle.apply(w["lq"], r["centroids"], r["gamma"], r["beta"], alpha=1.0)
    assert (a == r["assignments"]).all()
    x = w["lq"].astype(np.float64)
    np.testing.assert_allclose(out1, r["gamma"][a] * x + r["beta"][a], rtol=1e-13, atol=1e-13)
    out0, _ = oracle.apply(w["lq"], r["centroids"], r["gamma"], r["beta"], alpha=0.0)
    assert (out0 == x).all()
    outh, _ = oracle.apply(w["lq"], r["centroids"], r["gamma"], r["beta"], alpha=0.25)
    np.testing.assert_allclose(outh, 0.75 * x + 0.25 * out1, rtol=1e-12, atol=1e-12)
    # alpha = 1: the corrected cluster mean equals the FP cluster mean
    for k in range(4):
        if r["counts"][k]:
            np.testing.assert_allclose(out1[a == k].mean(axis=0), w["fp"][a == k].astype(np.float64).mean(axis=0),
                                       rtol=1e-9, atol=1e-9)


def test_seeded_fit_equals_fit_from_the_seeded_rows():
    w = workloads.planted_mixture(500, 6, 4, seed=14)
    idx = oracle.init_indices(500, 4, 77)
    r1 = oracle.fit(w["lq"], w["fp"], K=4, iters=5, seed=77)
    r2 = oracle.fit(w["lq"], w["fp"], K=4, iters=5, init_centroids=w["lq"][idx].astype(np.float64))
    for key in ("centroids", "gamma", "beta", "assignments", "inertia"):
        assert (r1[key] == r2[key]).all()
    r0 = oracle.fit(w["lq"], w["fp"], K=4, iters=0, seed=77)  # iters = 0: centroids are the init rows
    assert (r0["centroids"] == w["lq"][idx].astype(np.float64)).all() and len(r0["inertia"]) == 1
