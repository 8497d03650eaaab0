"""Pins for the checker's accept / correct / extra-token decision (oracle/spec_sampling.py).

None of these re-type the rule: they measure the law of the tokens the real decision
function commits and compare it with the target distribution (Sec. 1: the target's output
distribution is preserved exactly), or use cases whose answer is known without the rule.
"""
import numpy as np
import pytest

from oracle.spec_sampling import draw_index, greedy_accept, spec_accept

F32 = np.float32
TWO24 = 1 << 24


def _probs(rng, rows, V, sharp=1.5):
    z = rng.standard_normal((rows, V)) * sharp
    e = np.exp(z - z.max(axis=1, keepdims=True))
    return (e / e.sum(axis=1, keepdims=True)).astype(F32)


def _u(i):  # the i-th representable uniform
    return F32(i * 2.0 ** -24)


def _first_false(pred, lo=0, hi=TWO24):
    """Smallest i in [lo, hi] with pred(i) false, pred monotone true...true false...false."""
    while lo < hi:
        mid = (lo + hi) // 2
        if pred(mid):
            lo = mid + 1
        else:
            hi = mid
    return lo


def _draw_law(fn, V):
    """Exact law of x = fn(u) over the 2^24 uniforms, for fn non-decreasing in u."""
    law = np.zeros(V)
    start = 0
    for x in range(V):
        end = _first_false(lambda i: fn(_u(i)) <= x, start, TWO24)
        law[x] = (end - start) / TWO24
        start = end
    assert start == TWO24
    return law


@pytest.mark.parametrize("V,seed", [(5, 0), (16, 1), (11, 2)])
def test_k1_output_law_equals_target(V, seed):
    rng = np.random.default_rng(seed)
    p = _probs(rng, 2, V)
    q = _probs(rng, 1, V)
    law_first = np.zeros(V)
    law_bonus = np.zeros(V)
    acc_total = 0.0
    for d in range(V):
        # acceptance is monotone in the first uniform
        n_acc = _first_false(lambda i: spec_accept(p, q, [d], [_u(i), F32(0)])[0] == 1)
        f = n_acc / TWO24
        acc_total += float(q[0, d]) * f
        law_first[d] += float(q[0, d]) * f
        if n_acc < TWO24:
            rej_u = _u(TWO24 - 1)
            assert spec_accept(p, q, [d], [rej_u, F32(0)])[0] == 0
            law_first += float(q[0, d]) * (1 - f) * _draw_law(
                lambda us: spec_accept(p, q, [d], [rej_u, us])[1], V)
        if n_acc > 0:
            law_bonus += float(q[0, d]) * f * _draw_law(
                lambda us: spec_accept(p, q, [d], [_u(0), us])[1], V)
    # law of the first committed token is the target's first row
    np.testing.assert_allclose(law_first, p[0].astype(np.float64), atol=2e-6)
    # acceptance probability of position 1 is sum_x min(p, q)
    assert abs(acc_total - np.minimum(p[0], q[0]).astype(np.float64).sum()) < 2e-6
    # given acceptance, the extra token follows the last row (weights: P(accept, d))
    np.testing.assert_allclose(law_bonus / acc_total, p[1].astype(np.float64), atol=2e-6)


def test_k2_second_token_law():
    """Given that d_1 was accepted, the second committed token follows row 2 of the target."""
    V = 6
    rng = np.random.default_rng(7)
    p = _probs(rng, 3, V)
    q = _probs(rng, 2, V)
    d1 = int(np.argmax(np.minimum(p[0], q[0])))
    u1 = _u(0)  # always accepts d1 (ratio > 0)
    law = np.zeros(V)
    for d2 in range(V):
        n_acc = _first_false(lambda i: spec_accept(p, q, [d1, d2], [u1, _u(i), F32(0)])[0] == 2)
        f = n_acc / TWO24
        law[d2] += float(q[1, d2]) * f
        if n_acc < TWO24:
            rej = _u(TWO24 - 1)
            a, _ = spec_accept(p, q, [d1, d2], [u1, rej, F32(0)])
            assert a == 1
            law += float(q[1, d2]) * (1 - f) * _draw_law(
                lambda us: spec_accept(p, q, [d1, d2], [u1, rej, us])[1], V)
    np.testing.assert_allclose(law, p[1].astype(np.float64), atol=2e-6)


def test_first_rejection_stops_the_scan():
    """A rejected draft hides everything behind it, however acceptable."""
    V = 8
    rng = np.random.default_rng(3)
    p = _probs(rng, 4, V)
    q = p[:3].copy()
    q[1] = np.roll(p[1], 1)
    d = [0, int(np.argmin(p[1] / q[1])), 0]
    a, nxt = spec_accept(p, q, d, [F32(0.5), _u(TWO24 - 1), F32(0.0), F32(0.3)])
    assert a == 1
    assert nxt != d[1] or p[1, d[1]] > q[1, d[1]]


def test_q_equals_p_accepts_everything():
    rng = np.random.default_rng(11)
    V, k = 16, 5
    p = _probs(rng, k + 1, V)
    for trial in range(50):
        d = rng.integers(0, V, k)
        u = (rng.integers(0, TWO24, k + 1) * 2.0 ** -24).astype(F32)
        a, nxt = spec_accept(p, p[:k].copy(), d, u)
        assert a == k
        c = np.cumsum(p[k].astype(np.float64))
        # the extra token is the inverse CDF of the last row at u (up to the 2^-40 truncation)
        lo = 0.0 if nxt == 0 else c[nxt - 1] / c[-1]
        hi = c[nxt] / c[-1]
        assert lo - 1e-6 <= float(u[k]) <= hi + 1e-6


def test_draft_outside_target_support_is_rejected_and_resampled_from_p():
    V = 9
    rng = np.random.default_rng(5)
    p = _probs(rng, 2, V)
    p[0, 4] = 0.0
    p[0] /= p[0].sum(dtype=np.float64)
    p = p.astype(F32)
    q = np.zeros((1, V), dtype=F32)
    q[0, 4] = 1.0
    for i in (0, 1, TWO24 // 3, TWO24 - 1):
        assert spec_accept(p, q, [4], [_u(i), F32(0.2)])[0] == 0
    # residual = p exactly, so the correction follows p's own inverse CDF
    law = _draw_law(lambda us: spec_accept(p, q, [4], [_u(0), us])[1], V)
    np.testing.assert_allclose(law, p[0].astype(np.float64) / p[0].astype(np.float64).sum(), atol=2e-6)


def test_zero_draft_probability_with_positive_target_accepts():
    p = np.array([[0.5, 0.5], [1.0, 0.0]], dtype=F32)
    q = np.array([[1.0, 0.0]], dtype=F32)
    assert spec_accept(p, q, [1], [_u(TWO24 - 1), F32(0)]) == (1, 0)
    # 0/0 rejects; the residual is then p itself
    p2 = np.array([[1.0, 0.0], [1.0, 0.0]], dtype=F32)
    q2 = np.array([[1.0, 0.0]], dtype=F32)
    assert spec_accept(p2, q2, [1], [_u(0), F32(0.7)]) == (0, 0)


def test_residual_all_zero_falls_back_to_argmax():
    p = np.array([[0.25, 0.5, 0.25], [1, 0, 0]], dtype=F32)
    q = p[:1].copy()
    # force a rejection at equality is impossible (ratio = 1 > u), so test the draw directly
    assert draw_index(np.zeros(3, dtype=F32), F32(0.9), p[0]) == 1


def test_draw_index_is_the_integer_inverse_cdf():
    """Brute force with Python integers on every boundary of a small table."""
    w = np.array([0.125, 0.0, 0.5, 0.25, 0.0, 0.125], dtype=F32)
    edges = np.cumsum(w.astype(np.float64))
    for i in range(0, TWO24, 4099):
        u = i / TWO24
        expect = int(np.searchsorted(edges, u, side="right"))
        assert draw_index(w, _u(i), w) == expect
    for e in edges[:-1]:
        i = int(round(e * TWO24))
        assert draw_index(w, _u(i), w) == int(np.searchsorted(edges, e, side="right"))
        assert draw_index(w, _u(i - 1), w) == int(np.searchsorted(edges, e - 2.0 ** -24, side="right"))


def test_draw_index_never_lands_on_zero_weight():
    rng = np.random.default_rng(2)
    w = _probs(rng, 1, 64)[0]
    w[rng.integers(0, 64, 30)] = 0
    for i in rng.integers(0, TWO24, 2000):
        assert w[draw_index(w, _u(int(i)), w)] > 0


def test_greedy_is_longest_argmax_prefix_and_matches_onehot_rule():
    rng = np.random.default_rng(9)
    V, k = 12, 6
    for trial in range(40):
        z = rng.standard_normal((k + 1, V)).astype(F32)
        am = z.argmax(axis=1)
        d = am[:k].copy()
        cut = rng.integers(0, k + 1)
        if cut < k:
            d[cut] = (d[cut] + 1 + rng.integers(0, V - 1)) % V
        a, nxt = greedy_accept(z, d)
        assert a == cut and nxt == am[cut]
        # same outcome from the stochastic rule fed one-hot rows
        p = np.zeros((k + 1, V), dtype=F32)
        p[np.arange(k + 1), am] = 1
        q = np.zeros((k, V), dtype=F32)
        q[np.arange(k), d] = 1
        u = (rng.integers(0, TWO24, k + 1) * 2.0 ** -24).astype(F32)
        assert spec_accept(p, q, d, u) == (a, nxt)


def test_greedy_tie_takes_lowest_index():
    z = np.array([[1.0, 3.0, 3.0, 0.0], [2.0, 2.0, 2.0, 2.0]], dtype=F32)
    assert greedy_accept(z, [1]) == (1, 0)
    assert greedy_accept(z, [2]) == (0, 1)


def test_table7_accounting_each_pass_commits_accepted_plus_one():
    """Table 7: verification frequency = 1 / (mean draft length * acceptance rate + 1), i.e.
    each NAV pass commits accepted_len + 1 tokens."""
    import os
    rows = []
    with open(os.path.join(os.path.dirname(__file__), "golden", "table7_nav_statistics.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                name, freq, length, acc = line.split()
                rows.append((float(freq), float(length), float(acc)))
    assert len(rows) == 3
    for freq, length, acc in rows:
        assert abs(1.0 / (length * acc + 1.0) - freq) < 2e-4
