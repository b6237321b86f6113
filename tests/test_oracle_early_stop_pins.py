"""Pins of the oracle's early stop of the Lloyd loop (the paper fixes no stopping rule for k-means, Sec. 4, Setup):
a worked example by hand, the fixed-point property (stopping at the first repeated partition changes no output of
the full run), and the index of that pass found by brute force from full runs of every length."""
import numpy as np

import oracle


def test_worked_example_on_a_line():
    # points 0, 1, 10, 11 with initial centroids 0 and 1:
    #   pass 0: {0} {1, 10, 11}     objective 0 + 0 + 81 + 100 = 181,       means 0 and 22/3
    #   pass 1: {0, 1} {10, 11}     objective 0 + 1 + (8/3)^2 + (11/3)^2,   means 1/2 and 21/2
    #   pass 2: the same partition  objective 4 * 1/4 = 1                   -> stop
    x = np.array([[0.0], [1.0], [10.0], [11.0]], dtype=np.float32)
    init = np.array([[0.0], [1.0]])
    r = oracle.fit_early_stop(x, x, 2, 6, init_centroids=init)
    assert r["stable_at"] == 2
    assert r["assignments"].tolist() == [0, 0, 1, 1]
    np.testing.assert_allclose(r["centroids"], [[0.5], [10.5]], rtol=0, atol=0)
    np.testing.assert_allclose(r["inertia"], [181.0, 1.0 + 64.0 / 9 + 121.0 / 9, 1, 1, 1, 1, 1], rtol=1e-15)
    # too few passes to see a repeat
    assert oracle.fit_early_stop(x, x, 2, 1, init_centroids=init)["stable_at"] == -1
    assert oracle.fit_early_stop(x, x, 2, 0, init_centroids=init)["stable_at"] == -1
    # the repeat is seen by the final pass
    assert oracle.fit_early_stop(x, x, 2, 2, init_centroids=init)["stable_at"] == 2


def _mixture(seed, N, D, K, spread):
    rng = np.random.default_rng(seed)
    centres = rng.standard_normal((K, D)) * spread
    x = (centres[rng.integers(0, K, N)] + rng.standard_normal((N, D))).astype(np.float32)
    y = (1.1 * x + 0.05 * rng.standard_normal((N, D))).astype(np.float32)
    return x, y


def test_stopping_changes_no_output_of_the_full_run():
    seen = set()
    for seed, (N, D, K, spread, iters) in enumerate([(300, 5, 4, 6.0, 12), (500, 8, 6, 1.0, 5), (64, 3, 3, 3.0, 40),
                                                     (400, 6, 5, 0.5, 30), (50, 2, 1, 1.0, 4)]):
        x, y = _mixture(seed, N, D, K, spread)
        full = oracle.fit(x, y, K, iters, seed=seed)
        r = oracle.fit_early_stop(x, y, K, iters, seed=seed)
        for key in ("centroids", "gamma", "beta", "assignments", "counts"):
            assert (np.asarray(r[key]) == np.asarray(full[key])).all(), (seed, key)
        np.testing.assert_allclose(r["inertia"], full["inertia"], rtol=1e-13)
        seen.add(r["stable_at"] >= 0)
    assert seen == {True, False}  # both a run that stops and one that does not


def test_index_of_the_first_repeated_partition_by_brute_force():
    for seed in range(4):
        x, y = _mixture(10 + seed, 250, 4, 5, 2.0)
        iters = 25
        parts = [oracle.fit(x, y, 5, t, seed=seed)["assignments"] for t in range(iters + 1)]  # partition of pass t
        want = next((t for t in range(1, iters + 1) if (parts[t] == parts[t - 1]).all()), -1)
        assert oracle.fit_early_stop(x, y, 5, iters, seed=seed)["stable_at"] == want
