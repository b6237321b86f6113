"""Pins of the oracle's blending-coefficient sweep (the alpha display of Sec. 3.1; the ablation on alpha
in Sec. 5) against what the mathematics fixes: alpha = 0 is the uncorrected input, the squared error is
a parabola in alpha whose curvature is the energy of the correction term, a least-squares fit puts the
vertex at alpha = 1 with the residual variance as its value, Top-1 follows numpy's argmax of the
separately pinned inference, and a brute-force loop on tiny inputs."""
import numpy as np

import oracle


def _data(seed, N=300, D=11, K=3):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((N, D)).astype(np.float32) * 2
    y = (x * rng.uniform(0.5, 1.5, D) + rng.standard_normal((N, D)) * 0.4 + rng.standard_normal(D)).astype(np.float32)
    a = rng.integers(0, K, N).astype(np.int32)
    g = rng.uniform(0.3, 1.7, (K, D))
    b = rng.standard_normal((K, D))
    return x, y, a, g, b


def test_alpha_zero_is_the_uncorrected_input():
    x, y, a, g, b = _data(1)
    lab = np.argmax(y, axis=1).astype(np.int32)
    r = oracle.alpha_sweep(x, a, g, b, [0.0], fp=y, labels=lab)
    assert (r["top1"][:, 0] == np.argmax(x, axis=1)).all()
    assert r["hits"][0] == int((np.argmax(x, axis=1) == lab).sum())
    d = x.astype(np.float64) - y.astype(np.float64)
    np.testing.assert_allclose(r["sq_err"][0], (d * d).sum(), rtol=1e-12)
    xs = np.sort(x.astype(np.float64), axis=1)
    np.testing.assert_allclose(r["margin"][:, 0], xs[:, -1] - xs[:, -2], rtol=0, atol=0)


def test_squared_error_is_a_parabola_with_the_energy_of_the_correction_as_curvature():
    x, y, a, g, b = _data(2)
    h = 0.25
    al = [-0.5, -0.5 + h, -0.5 + 2 * h, 0.9, 1.7]
    sq = oracle.alpha_sweep(x, a, g, b, al, fp=y)["sq_err"]
    x64 = x.astype(np.float64)
    corr = x64 * (g[a] - 1.0) + b[a]  # the term alpha multiplies
    base = x64 - y.astype(np.float64)
    s_bb, s_ab, s_aa = (corr * corr).sum(), (base * corr).sum(), (base * base).sum()
    np.testing.assert_allclose(sq[0] - 2 * sq[1] + sq[2], 2 * h * h * s_bb, rtol=1e-9)
    for t, v in zip(al, sq):
        np.testing.assert_allclose(v, s_aa + 2 * t * s_ab + t * t * s_bb, rtol=1e-11)


def test_least_squares_parameters_put_the_vertex_at_alpha_one():
    x, y, a, _, _ = _data(3, N=600, D=7, K=4)
    x64, y64 = x.astype(np.float64), y.astype(np.float64)
    K, D = 4, x.shape[1]
    g = np.empty((K, D))
    b = np.empty((K, D))
    resid = 0.0
    for k in range(K):
        m = a == k
        for j in range(D):
            slope, icpt = np.polyfit(x64[m, j], y64[m, j], 1)  # library least squares
            g[k, j], b[k, j] = slope, icpt
            c = np.cov(x64[m, j], y64[m, j], bias=True)
            resid += m.sum() * (c[1, 1] - c[0, 1] ** 2 / c[0, 0])
    t = 0.37
    sq = oracle.alpha_sweep(x, a, g, b, [1.0, 1.0 - t, 1.0 + t, 0.0], fp=y)["sq_err"]
    np.testing.assert_allclose(sq[0], resid, rtol=1e-9)
    np.testing.assert_allclose(sq[1], sq[2], rtol=1e-9)  # symmetric about the vertex
    assert sq[0] < sq[1] and sq[0] < sq[3]
    # and the oracle's own fit produces those parameters
    ga, ba, _ = oracle.affine(x, y, a, K)
    np.testing.assert_allclose(ga, g, rtol=1e-8, atol=1e-10)
    np.testing.assert_allclose(ba, b, rtol=1e-8, atol=1e-9)


def test_top1_is_argmax_of_the_inference_output():
    rng = np.random.default_rng(4)
    N, D, K = 400, 9, 5
    cent = rng.standard_normal((K, D)) * 3
    x = (cent[rng.integers(0, K, N)] + rng.standard_normal((N, D))).astype(np.float32)
    g = rng.uniform(0.2, 1.8, (K, D))
    b = rng.standard_normal((K, D)) * 2
    lab = rng.integers(0, D, N).astype(np.int32)
    for alpha in (0.3, 1.0):
        out, a = oracle.apply(x, cent, g, b, alpha)
        r = oracle.alpha_sweep(x, a, g, b, [alpha], labels=lab)
        assert (r["top1"][:, 0] == np.argmax(out, axis=1)).all()
        assert r["hits"][0] == int((np.argmax(out, axis=1) == lab).sum())
        so = np.sort(out, axis=1)
        np.testing.assert_allclose(r["margin"][:, 0], so[:, -1] - so[:, -2], rtol=1e-12, atol=1e-13)
        assert (r["sq_err"] == 0).all()


def test_brute_force_on_tiny_inputs_with_ties_and_outside_labels():
    x = np.array([[1.0, 3.0, 3.0], [2.0, -1.0, 0.5], [0.0, 0.0, 0.0], [5.0, 4.0, 6.0], [1.0, 2.0, 0.0]], dtype=np.float32)
    y = np.array([[0.5, 2.0, 4.0], [1.0, 1.0, 1.0], [0.0, 1.0, 0.0], [6.0, 4.0, 5.0], [1.0, 1.0, 1.0]], dtype=np.float32)
    g = np.array([[1.5, 1.0, 1.0], [0.5, 3.0, 1.0]])
    b = np.array([[0.0, 0.0, 0.0], [1.0, 0.0, -2.0]])
    a = np.array([0, 1, 1, 7, -1], dtype=np.int32)  # 7 and -1: no cluster, the row stays as it is
    lab = np.array([1, 0, 0, 2, 1], dtype=np.int32)
    al = [0.0, 0.5, 1.0, 2.0]
    r = oracle.alpha_sweep(x, a, g, b, al, fp=y, labels=lab)
    for s, alpha in enumerate(al):
        hits, err = 0, 0.0
        for i in range(5):
            row = []
            for j in range(3):
                q = float(x[i, j])
                c = q
                if 0 <= a[i] < 2:
                    c = q + alpha * (g[a[i], j] * q + b[a[i], j] - q)
                row.append(c)
                err += (c - float(y[i, j])) ** 2
            top = max(row)
            arg = row.index(top)  # first position of the maximum
            rest = sorted(row)[-2]
            assert r["top1"][i, s] == arg
            assert abs(r["margin"][i, s] - (top - rest)) < 1e-15
            hits += int(arg == lab[i])
        assert r["hits"][s] == hits
        assert abs(r["sq_err"][s] - err) < 1e-12
    # row 0 ties entries 1 and 2 at every alpha (gamma = 1, beta = 0 there): the first one wins
    assert (r["top1"][0] == 1).all() and (r["margin"][0] == 0).all()
    # rows without a cluster never move
    assert (r["top1"][3] == 2).all() and (r["top1"][4] == 1).all()


def test_single_channel_rows():
    x = np.array([[1.0], [-2.0]], dtype=np.float32)
    r = oracle.alpha_sweep(x, np.zeros(2, np.int32), np.array([[2.0]]), np.array([[1.0]]), [1.0], fp=x, labels=np.zeros(2, np.int32))
    assert (r["top1"] == 0).all() and np.isinf(r["margin"]).all() and r["hits"][0] == 2
    np.testing.assert_allclose(r["sq_err"][0], (3.0 - 1.0) ** 2 + (-3.0 + 2.0) ** 2)
