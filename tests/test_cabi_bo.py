"""The library's autotuner functions (host arithmetic, no GPU) against the checker (oracle/bo.py), and
the whole tuning loop on a synthetic time-per-accepted-token objective built from the library's own
trigger and batching functions (the paper's objective needs its testbed; Sec. 3.3, appendix on BO)."""
import numpy as np
import pytest

from oracle import bo
from paper_2605_13319_amd import inputs as I
from paper_2605_13319_amd import nav


def test_posterior_equals_the_checker():
    rng = np.random.default_rng(11)
    for n, l, noise in ((1, 0.3, 1e-6), (2, 0.3, 0.0), (7, 0.2, 1e-6), (16, 0.3, 1e-4), (40, 0.5, 1e-3)):
        x = rng.random((n, 2))
        y = 130 + 20 * rng.standard_normal(n)
        q = np.concatenate([rng.random((30, 2)), x[:3]])
        mu, sd = nav.bo_posterior(x, y, l, noise, q)
        mu_ref, sd_ref = bo.posterior(x, y, l, noise, q)
        assert np.allclose(mu, mu_ref, rtol=0, atol=1e-8 * max(1.0, y.std())), n
        assert np.allclose(sd, sd_ref, rtol=0, atol=1e-6 * max(1.0, y.std())), n
    # all observations equal: scale 1, posterior mean is that value everywhere
    mu, sd = nav.bo_posterior([[0.1, 0.1], [0.9, 0.9]], [5.0, 5.0], 0.3, 1e-6, [[0.5, 0.5]])
    assert abs(mu[0] - 5.0) < 1e-12 and 0 < sd[0] <= 1.0


def test_suggestion_equals_the_checker():
    rng = np.random.default_rng(12)
    for n in (1, 2, 5, 9, 15):
        x = rng.random((n, 2))
        y = 130 + 20 * rng.standard_normal(n)
        for g in (4, 16, 33):
            nxt, ei = nav.bo_suggest(x, y, 0.3, 1e-6, 0.1, g)
            nxt_ref, ei_ref = bo.suggest(x, y, 0.3, 1e-6, 0.1, g)
            assert abs(ei - ei_ref) <= 1e-9 * max(1.0, ei_ref), (n, g)
            if nxt != nxt_ref:  # two raster points within rounding of each other: both must be maximisers
                ys, _, _ = bo.standardise(y)
                m, s = bo.posterior(x, ys, 0.3, 1e-6, [nxt])
                assert abs(bo.expected_improvement(m, s, float(ys.min()), 0.1)[0] - ei_ref) <= 1e-9, (n, g)


def test_argument_errors():
    x, y = [[0.2, 0.2], [0.4, 0.9]], [1.0, 2.0]
    for bad in (lambda: nav.bo_suggest(x, y, 0.0, 1e-6, 0.1, 8), lambda: nav.bo_suggest(x, y, 0.3, -1.0, 0.1, 8),
                lambda: nav.bo_suggest(x, y, 0.3, 1e-6, -0.1, 8), lambda: nav.bo_suggest(x, y, 0.3, 1e-6, 0.1, 0),
                lambda: nav.bo_suggest(x, [1.0, float("nan")], 0.3, 1e-6, 0.1, 8),
                lambda: nav.bo_suggest([[0.2, 0.2], [0.2, 0.2]], y, 0.3, 0.0, 0.1, 8),  # same point twice, no noise
                lambda: nav.bo_posterior(x, y, float("inf"), 1e-6, [[0.5, 0.5]])):
        with pytest.raises(nav.PipesdError) as e:
            bad()
        assert e.value.status == nav.EINVAL
    assert nav._lib.pipesd_bo_suggest(None, None, 1, 0.3, 1e-6, 0.1, 8, None, None) == nav.EINVAL


def synthetic_tpt(alpha, beta, gamma, t_nav, n_conf=6000, seed=77):
    """Time per accepted token of a simulated edge/cloud loop as a function of (R1, R2): a seeded
    stream of draft confidences is cut into rounds by the dual-threshold trigger; draft i of a round
    is accepted iff a seeded uniform lies below its confidence, the accepted prefix plus one token is
    committed; a round costs the optimal pipelined upload time of its drafts plus one NAV."""
    conf = I.make_confidences(n_conf, seed)
    u = np.random.default_rng(seed + 1).random(n_conf)
    t_cache = {}

    def f(r1, r2):
        lengths, used = nav.trigger_rounds(conf, r1, r2, 16)
        total, committed, pos = 0.0, 0, 0
        for n in lengths:
            if n not in t_cache:
                t_cache[n] = nav.batching_optimal(n, alpha, beta, gamma)[1]
            total += t_cache[n] + t_nav
            a = 0
            while a < n and u[pos + a] < conf[pos + a]:
                a += 1
            committed += a + 1
            pos += n
        return total / max(committed, 1)
    return f


def test_tuning_loop_equals_the_checker_and_beats_the_coarse_grid():
    f = synthetic_tpt(alpha=20.0, beta=4.0, gamma=25.0, t_nav=40.0)
    first = tuple(np.random.default_rng(5).random(2))  # the one random initial sample
    xs, ys = [first], [f(*first)]
    while len(xs) < 16:
        nxt, _ = nav.bo_suggest(xs, ys, 0.3, 1e-4, 0.1, 32)
        xs.append(nxt)
        ys.append(f(*nxt))
    xs_ref, ys_ref, best_ref = bo.tune(f, first, 16, 0.3, 1e-4, 0.1, 32)
    assert xs == xs_ref and ys == ys_ref
    best = min(ys)
    coarse = min(f((i + 0.5) / 4, (j + 0.5) / 4) for i in range(4) for j in range(4))  # 16 points of a 4 x 4 grid
    dense = min(f((i + 0.5) / 32, (j + 0.5) / 32) for i in range(32) for j in range(32))
    print(f"TPT: autotuner {best:.2f}, 4x4 grid {coarse:.2f}, dense optimum {dense:.2f}, first sample {ys[0]:.2f}")
    assert best <= coarse + 1e-9 and best <= 1.03 * dense
