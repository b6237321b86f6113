"""Pins of the oracle's D^2-weighted seeding (k-means++, Arthur and Vassilvitskii 2007): a plain Python
re-statement of the published procedure on small inputs, the sampling frequencies the procedure prescribes on
a three-point example, one seed per planted cluster when the clusters are far apart, degenerate inputs, and
the uniform draws against the published SplitMix64 stream."""
import numpy as np

import oracle


def _uniform(seed, t):
    return (oracle.splitmix64(seed, t) >> 11) * 2.0 ** -53


def _by_hand(x, K, seed):
    """the procedure written out with Python floats (IEEE double) and loops"""
    N = len(x)
    idx = [min(int(_uniform(seed, 0) * N), N - 1)]
    d2 = None
    for t in range(1, K + 1):
        c = x[idx[-1]]
        new = [sum((float(a) - float(b)) ** 2 for a, b in zip(row, c)) for row in x]
        d2 = new if d2 is None else [min(p, q) for p, q in zip(d2, new)]
        if t == K:
            break
        total = 0.0
        for v in d2:
            total += v
        pick = None
        if total > 0.0:
            target = _uniform(seed, t) * total
            run = 0.0
            for i, v in enumerate(d2):
                run += v
                if run > target:
                    pick = i
                    break
        if pick is None:
            pick = min(i for i in range(N) if i not in idx)
        idx.append(pick)
    return idx


def test_uniform_draws_come_from_the_published_stream():
    # first outputs of SplitMix64 seeded with 1234567 (the reference vectors of the generator's authors)
    assert oracle.splitmix64(1234567, 0) == 6457827717110365317
    assert oracle.splitmix64(1234567, 1) == 3203168211198807973
    u = _uniform(1234567, 0)
    assert 0.0 <= u < 1.0 and u == (6457827717110365317 >> 11) / 2.0 ** 53


def test_matches_the_procedure_written_out_by_hand():
    rng = np.random.default_rng(0)
    for seed in range(12):
        N, D, K = int(rng.integers(5, 40)), int(rng.integers(1, 6)), int(rng.integers(1, 5))
        x = rng.standard_normal((N, D)).astype(np.float32)
        got = oracle.kmeanspp(x, K, seed=seed)
        assert list(got) == _by_hand(x.tolist(), K, seed), seed
        assert len(set(got.tolist())) == K


def test_second_draw_follows_the_squared_distances():
    """three points on a line at 0, 1 and 3: given the first centre, the two others are drawn in proportion to
    their squared distances to it (1 : 9 from 0, 1 : 4 from 1, 9 : 4 from 3)"""
    x = np.array([[0.0], [1.0], [3.0]], dtype=np.float32)
    counts = {0: [0, 0, 0], 1: [0, 0, 0], 2: [0, 0, 0]}
    for seed in range(6000):
        a, b = oracle.kmeanspp(x, 2, seed=seed)
        counts[int(a)][int(b)] += 1
    n0, n1, n2 = (sum(counts[i]) for i in range(3))
    assert min(n0, n1, n2) > 1800  # the first draw is uniform
    assert counts[0][0] == counts[1][1] == counts[2][2] == 0  # a centre is at distance 0 from itself
    assert abs(counts[0][2] / n0 - 9 / 10) < 0.03
    assert abs(counts[1][2] / n1 - 4 / 5) < 0.03
    assert abs(counts[2][0] / n2 - 9 / 13) < 0.04


def test_far_apart_clusters_get_one_seed_each():
    rng = np.random.default_rng(3)
    K, per, D = 6, 50, 4
    centres = rng.standard_normal((K, D)) * 1000.0
    lab = np.repeat(np.arange(K), per)
    x = (centres[lab] + rng.standard_normal((K * per, D))).astype(np.float32)
    for seed in range(20):
        idx = oracle.kmeanspp(x, K, seed=seed)
        assert sorted(lab[idx].tolist()) == list(range(K)), seed


def test_degenerate_inputs():
    same = np.ones((6, 3), dtype=np.float32)
    idx = oracle.kmeanspp(same, 4, seed=5)
    first = int(idx[0])
    rest = [i for i in range(6) if i != first][:3]
    assert idx.tolist() == [first] + rest  # zero total weight: lowest rows not chosen yet
    # two distinct values: the second centre must be a row of the other value, the third falls back
    x = np.array([[0.0], [0.0], [5.0], [5.0]], dtype=np.float32)
    for seed in range(10):
        idx = oracle.kmeanspp(x, 3, seed=seed)
        assert x[idx[0], 0] != x[idx[1], 0]
        assert idx[2] == min(i for i in range(4) if i not in idx[:2].tolist())
    assert oracle.kmeanspp(x, 1, seed=9).shape == (1,)
    assert sorted(oracle.kmeanspp(x, 4, seed=2).tolist()) == [0, 1, 2, 3]


def test_best_of_several_runs_is_one_of_the_single_runs_and_none_is_better():
    """fit_restarts is a selection among fit runs: its result must be, field by field, the single run of the seed it
    names, that run must have the lowest final objective, and the objective must be what scipy's distance routine
    gives for the returned partition"""
    from scipy.spatial.distance import cdist
    rng = np.random.default_rng(8)
    K, D = 5, 6
    centres = rng.standard_normal((K, D)) * 2.5
    x = (centres[rng.integers(0, K, 400)] + rng.standard_normal((400, D))).astype(np.float32)
    y = (x * 0.8 + 0.1 * rng.standard_normal((400, D))).astype(np.float32)
    for pp in (False, True):
        r = oracle.fit_restarts(x, y, K, 6, seed=20, restarts=7, kmeanspp_seeding=pp)
        b = int(r["best_run"])
        init = x[oracle.kmeanspp(x, K, seed=20 + b)].astype(np.float64) if pp else None
        single = oracle.fit(x, y, K, 6, seed=20 + b, init_centroids=init)
        for key in ("centroids", "gamma", "beta", "assignments", "counts", "inertia"):
            assert (np.asarray(r[key]) == np.asarray(single[key])).all(), key
        finals = r["final_inertia"]
        assert finals.shape == (7,) and b == int(np.argmin(finals)) and finals[b] == r["inertia"][-1]
        d = cdist(x.astype(np.float64), r["centroids"], "sqeuclidean")
        np.testing.assert_allclose(finals[b], d[np.arange(400), r["assignments"]].sum(), rtol=1e-12)
        assert (r["assignments"] == d.argmin(axis=1)).all()
    # the runs do differ on this input: the selection is not vacuous
    assert len(set(np.round(oracle.fit_restarts(x, y, K, 6, seed=20, restarts=7)["final_inertia"], 6))) > 1
