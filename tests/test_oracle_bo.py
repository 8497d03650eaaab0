"""Pins of the autotuner's checker (oracle/bo.py; Sec. 3.3 and the appendix on BO): kernel values
from the Matern 5/2 formula, Gaussian-process identities, scikit-learn's GP regressor as an
independent library witness, Expected Improvement against its defining integral."""
import math

import numpy as np
import pytest

from oracle import bo


def test_matern52_known_values_and_symmetry():
    a = np.array([[0.2, 0.3]])
    assert bo.matern52(a, a, 0.4)[0, 0] == 1.0
    # at distance = length scale: (1 + sqrt5 + 5/3) exp(-sqrt5)
    b = np.array([[0.2 + 0.4, 0.3]])
    want = (1 + math.sqrt(5) + 5 / 3) * math.exp(-math.sqrt(5))
    assert abs(bo.matern52(a, b, 0.4)[0, 0] - want) < 1e-15 and abs(want - 0.523994) < 1e-6
    # only the Euclidean distance matters, in both coordinates
    c = np.array([[0.2, 0.3 - 0.4]])
    d = np.array([[0.2 + 0.4 / math.sqrt(2), 0.3 + 0.4 / math.sqrt(2)]])
    assert abs(bo.matern52(a, c, 0.4)[0, 0] - want) < 1e-15 and abs(bo.matern52(a, d, 0.4)[0, 0] - want) < 1e-14
    pts = np.random.default_rng(1).random((7, 2))
    K = bo.matern52(pts, pts, 0.3)
    assert np.allclose(K, K.T) and np.all(np.linalg.eigvalsh(K) > 0)
    # twice differentiable at 0: k(r) = 1 - (5/6)(r/l)^2 + O(r^4)
    r = 1e-4
    assert abs(bo.matern52(a, a + [[r, 0]], 1.0)[0, 0] - (1 - 5 / 6 * r * r)) < 1e-11


def test_posterior_interpolates_and_reverts_to_the_mean():
    rng = np.random.default_rng(2)
    x = rng.random((6, 2))
    y = 100 + 30 * rng.standard_normal(6)
    mu, sd = bo.posterior(x, y, 0.3, 1e-12, x)
    assert np.allclose(mu, y, atol=1e-6) and np.all(sd < 1e-4 * y.std())
    far = np.array([[50.0, 50.0]])
    mu, sd = bo.posterior(x, y, 0.3, 1e-12, far)
    assert abs(mu[0] - y.mean()) < 1e-9 and abs(sd[0] - y.std()) < 1e-9
    # shifting and scaling the observations shifts and scales the posterior
    q = rng.random((5, 2))
    m1, s1 = bo.posterior(x, y, 0.3, 1e-6, q)
    m2, s2 = bo.posterior(x, 7 * y - 3, 0.3, 1e-6, q)
    assert np.allclose(m2, 7 * m1 - 3) and np.allclose(s2, 7 * s1)


def test_posterior_two_points_closed_form():
    """Two observations, no noise: standardised values are +1 and -1, so by symmetry
    mu_s(q) = (k1 - k2) / (1 - rho) and var_s = 1 - (k1^2 + k2^2 - 2 rho k1 k2) / (1 - rho^2)."""
    x = np.array([[0.2, 0.5], [0.7, 0.5]])
    y = np.array([130.0, 150.0])  # mean 140, population std 10
    q = np.array([[0.4, 0.6]])
    l = 0.35
    k = lambda a, b: float(bo.matern52(np.array([a]), np.array([b]), l)[0, 0])
    rho, k1, k2 = k(x[0], x[1]), k(x[0], q[0]), k(x[1], q[0])
    mu_s = (-k1 + k2) / (1 - rho)  # y_s = (-1, +1)
    var_s = 1 - (k1 * k1 + k2 * k2 - 2 * rho * k1 * k2) / (1 - rho * rho)
    mu, sd = bo.posterior(x, y, l, 0.0, q)
    assert abs(mu[0] - (140 + 10 * mu_s)) < 1e-10 and abs(sd[0] - 10 * math.sqrt(var_s)) < 1e-10


def test_posterior_matches_scikit_learn():
    sk = pytest.importorskip("sklearn.gaussian_process")
    from sklearn.gaussian_process.kernels import Matern
    rng = np.random.default_rng(3)
    for n, l, noise in ((1, 0.3, 1e-6), (5, 0.3, 1e-6), (12, 0.15, 1e-3), (16, 0.5, 1e-2)):
        x = rng.random((n, 2))
        y = 120 + 25 * rng.standard_normal(n)
        q = rng.random((40, 2))
        ys, mean, scale = bo.standardise(y)
        gp = sk.GaussianProcessRegressor(kernel=Matern(length_scale=l, nu=2.5), alpha=noise, optimizer=None)
        gp.fit(x, ys)
        m_ref, s_ref = gp.predict(q, return_std=True)
        mu, sd = bo.posterior(x, y, l, noise, q)
        assert np.allclose(mu, mean + scale * m_ref, atol=1e-8 * scale), n
        assert np.allclose(sd, scale * s_ref, atol=1e-6 * scale), n


def test_expected_improvement_against_its_integral_and_limits():
    # EI = E[max(best - xi - Y, 0)], Y ~ N(mu, s^2): plain quadrature of the definition
    for mu, s, best, xi in ((0.3, 0.5, -0.2, 0.1), (-1.0, 0.2, -0.5, 0.1), (0.0, 1.0, 0.0, 0.0), (2.0, 0.7, -1.0, 0.1)):
        t = np.linspace(mu - 12 * s, mu + 12 * s, 400001)
        integrand = np.maximum(best - xi - t, 0.0) * np.exp(-0.5 * ((t - mu) / s) ** 2) / (s * math.sqrt(2 * math.pi))
        want = float(np.sum(0.5 * (integrand[1:] + integrand[:-1]) * np.diff(t)))
        got = bo.expected_improvement(np.array([mu]), np.array([s]), best, xi)[0]
        assert abs(got - want) < 1e-8, (mu, s, best, xi)
    # no uncertainty: the improvement itself, or nothing
    assert bo.expected_improvement(np.array([-1.0, 1.0]), np.array([0.0, 0.0]), 0.0, 0.1).tolist() == [0.9, 0.0]
    # mean exactly at best - xi: s / sqrt(2 pi)
    assert abs(bo.expected_improvement(np.array([0.4]), np.array([0.3]), 0.5, 0.1)[0] - 0.3 / math.sqrt(2 * math.pi)) < 1e-15
    # more uncertainty never lowers EI; a larger xi never raises it
    s = np.linspace(0.01, 2, 50)
    e = bo.expected_improvement(np.full(50, 0.2), s, 0.0, 0.1)
    assert np.all(np.diff(e) > 0)
    assert bo.expected_improvement(np.array([0.2]), np.array([0.5]), 0.0, 0.3)[0] < e[np.argmin(abs(s - 0.5))] + 1e-3


def test_suggest_and_tune_on_a_smooth_bowl():
    g = 16
    pts = bo.grid_points(g)
    assert pts.shape == (256, 2) and pts[0].tolist() == [1 / 32, 1 / 32] and pts[1].tolist() == [1 / 32, 3 / 32]
    # one observation: the kernel depends on the distance alone, so EI grows with it and the grid
    # point farthest from the sample is suggested
    nxt, ei = bo.suggest([[0.1, 0.2]], [5.0], 0.3, 1e-6, 0.1, g)
    assert nxt == (31 / 32, 31 / 32) and ei > 0
    f = lambda r1, r2: 100 + 80 * (r1 - 0.62) ** 2 + 50 * (r2 - 0.3) ** 2
    xs, ys, best = bo.tune(f, (0.9, 0.9), 16, 0.3, 1e-6, 0.1, g)
    assert len(xs) == 16 and len(set(xs)) == 16  # never the same point twice: EI vanishes at an observed point
    grid_best = min(f(*p) for p in pts)
    assert ys[best] - grid_best < 0.5 and ys[best] < f(0.9, 0.9) - 5
