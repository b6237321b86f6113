"""Pins of the oracle's Lloyd loop with distance bounds (Hamerly, SDM 2010; the paper fixes no k-means variant,
Sec. 4, Setup).  What defines the method: it returns exactly what the plain loop returns, whatever it leaves out.
Pinned by that identity on inputs that settle, inputs that keep moving, duplicates, empty clusters and exact ties,
by a sweep of small random cases, by a worked example of the bounds on a line, and by checks on the number of rows
it evaluates (never fewer than the rows that actually change cluster; none once a separated mixture has settled)."""
import numpy as np

import oracle


def _mixture(seed, N, D, K, spread):
    rng = np.random.default_rng(seed)
    centres = rng.standard_normal((K, D)) * spread
    x = (centres[rng.integers(0, K, N)] + rng.standard_normal((N, D))).astype(np.float32)
    y = (1.1 * x + 0.05 * rng.standard_normal((N, D))).astype(np.float32)
    return x, y


def _same_as_fit(x, y, K, iters, **kw):
    full = oracle.fit(x, y, K, iters, **kw)
    r = oracle.fit_bounds(x, y, K, iters, **kw)
    for key in ("centroids", "gamma", "beta", "assignments", "counts"):
        assert (np.asarray(r[key]) == np.asarray(full[key])).all(), key
    assert r["evaluated"].shape == (iters + 1,) and r["evaluated"][0] == len(x)
    return r


def test_worked_example_on_a_line():
    # points 0, 1, 10, 11, initial centroids 0 and 10.
    #   pass 0 (all four rows): clusters {0, 1} {10, 11}; u = 0, 1, 0, 1; l = 10, 9, 10, 9
    #   update: centroids 1/2 and 21/2, both move by 1/2: u = 1/2, 3/2, 1/2, 3/2; l = 19/2, 17/2, 19/2, 17/2;
    #   half the distance between the centroids is 5: every row has u < max(5, l), none is evaluated
    #   later updates move nothing
    x = np.array([[0.0], [1.0], [10.0], [11.0]], dtype=np.float32)
    r = oracle.fit_bounds(x, x, 2, 3, init_centroids=np.array([[0.0], [10.0]]))
    assert r["evaluated"].tolist() == [4, 0, 0, 0]
    assert r["assignments"].tolist() == [0, 0, 1, 1]
    assert r["centroids"].tolist() == [[0.5], [10.5]]
    # initial centroids 0 and 1: pass 0 gives {0} {1, 10, 11}, u = 0, 0, 9, 10, l = 1, 1, 10, 11.  The update moves
    # centroid 1 from 1 to 22/3 (by 19/3) and centroid 0 not at all: u = 0, 19/3, 46/3, 49/3;
    # l = 1 - 19/3 < 0 for row 0 and 1, 10, 11 for rows 1, 2, 3 (their own centroid is the one that moved most, the
    # other moved by 0); half the distance between the centroids is 11/3.
    #   row 0: u = 0 < 11/3: left alone.   row 1: 19/3 < max(11/3, 1) fails; tightened u = |1 - 22/3| = 19/3 fails
    #   again: evaluated (it moves to cluster 0).   row 2: 46/3 < 10 fails; tightened u = 8/3 < 10: left alone.
    #   row 3: 49/3 < 11 fails; tightened u = 11/3 < 11: left alone.        -> one row evaluated in pass 1
    r = oracle.fit_bounds(x, x, 2, 1, init_centroids=np.array([[0.0], [1.0]]))
    assert r["evaluated"].tolist() == [4, 1]
    assert r["assignments"].tolist() == [0, 0, 1, 1]


def test_same_result_as_the_plain_loop():
    for seed, (N, D, K, spread, iters) in enumerate([(300, 5, 4, 6.0, 12), (500, 8, 6, 1.0, 8), (64, 3, 3, 3.0, 30),
                                                     (400, 6, 5, 0.5, 25), (50, 2, 1, 1.0, 4), (40, 2, 40, 1.0, 3),
                                                     (700, 16, 12, 0.3, 15)]):
        x, y = _mixture(seed, N, D, K, spread)
        _same_as_fit(x, y, K, iters, seed=seed)


def test_duplicates_empty_clusters_and_exact_ties():
    rng = np.random.default_rng(3)
    base = rng.integers(-3, 4, (6, 4)).astype(np.float32)   # small integers: distances are exact, ties are exact
    x = np.repeat(base, 30, axis=0)
    y = (2 * x + 1).astype(np.float32)
    for K in (2, 5, 9):
        for seed in range(4):
            _same_as_fit(x, y, K, 6, seed=seed)
    # a row at the exact midpoint of two centroids must go to the lower index, also when a bound would allow it to
    # stay: the strict comparisons decide
    x = np.array([[0.0], [2.0], [4.0], [4.0], [8.0]], dtype=np.float32)
    for init in ([[0.0], [4.0]], [[4.0], [0.0]], [[2.0], [6.0]], [[8.0], [0.0]]):
        _same_as_fit(x, x, 2, 5, init_centroids=np.array(init))


def test_sweep_of_small_random_cases():
    rng = np.random.default_rng(11)
    for case in range(120):
        N = int(rng.integers(8, 80))
        D = int(rng.integers(1, 6))
        K = int(rng.integers(1, min(N, 9) + 1))
        iters = int(rng.integers(0, 12))
        # coarse grid values: many exact ties and repeated rows
        x = rng.integers(-4, 5, (N, D)).astype(np.float32) * (0.5 if case % 2 else 1.0)
        y = rng.standard_normal((N, D)).astype(np.float32)
        _same_as_fit(x, y, K, iters, seed=case)


def test_rows_that_change_cluster_are_always_evaluated():
    x, y = _mixture(2, 600, 6, 7, 0.8)
    iters = 15
    r = _same_as_fit(x, y, 7, iters, seed=5)
    cent = x[oracle.init_indices(len(x), 7, 5)].astype(np.float64)
    prev = None
    for t in range(iters + 1):
        a = oracle.assign(x, cent)
        if prev is not None:
            assert r["evaluated"][t] >= int((a != prev).sum())
        if t < iters:
            cent, _ = oracle.update(x, a, cent)
        prev = a
    assert (r["evaluated"][1:] < len(x)).all()   # and the bounds do leave rows out


def test_a_settled_separated_mixture_is_not_evaluated_again():
    rng = np.random.default_rng(4)
    centres = np.array([[0.0, 0.0], [40.0, 0.0], [0.0, 40.0], [40.0, 40.0]])
    lab = rng.integers(0, 4, 400)
    x = (centres[lab] + rng.standard_normal((400, 2))).astype(np.float32)
    init = centres + 1.0
    r = _same_as_fit(x, x, 4, 6, init_centroids=init)
    assert (r["assignments"] == lab).all()
    assert r["evaluated"].tolist() == [400, 0, 0, 0, 0, 0, 0]
