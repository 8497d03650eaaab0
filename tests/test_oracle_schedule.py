"""Pins of the scheduling checker (oracle/schedule.py): values worked out by hand from Eqs. (1)-(6),
closed forms, bounds that hold for every batching, recurrence (7) of the optimality proof, and
the trigger rule of Sec. 3.3 on sequences small enough to follow on paper."""
import functools
import math

import numpy as np
import pytest

from oracle import schedule as S


# ---- Eqs. (1)-(6), by hand --------------------------------------------------------------------
# N = 4, alpha = 3, beta = 1, gamma = 2: generation of token j ends at 2 j.
#   (1)        one batch of 4: sent 8 -> 8 + 3 + 4                                  = 15
#   (1,3)      {1,2} sent 4 -> 9; {3,4} ready 8, link free 9 -> 9 + 5               = 14
#   (1,2)      {1} 2 -> 6; {2,3,4} ready 8 -> 8 + 6                                 = 14
#   (1,4)      {1,2,3} 6 -> 12; {4} ready 8, free 12 -> 12 + 4                      = 16
#   (1,2,3)    2 -> 6; 6 -> 10; {3,4} ready 8, free 10 -> 10 + 5                    = 15
#   (1,2,4)    2 -> 6; {2,3} ready 6 -> 11; {4} ready 8, free 11 -> 15              = 15
#   (1,3,4)    4 -> 9; {3} ready 6, free 9 -> 13; {4} ready 8, free 13 -> 17        = 17
#   (1,2,3,4)  2 -> 6; 6 -> 10; 10 -> 14; 14 -> 18                                  = 18
HAND_N4 = {(1,): 15, (1, 3): 14, (1, 2): 14, (1, 4): 16, (1, 2, 3): 15, (1, 2, 4): 15, (1, 3, 4): 17, (1, 2, 3, 4): 18}


def test_pipeline_time_of_every_batching_of_four_tokens():
    seen = set()
    for b in S.all_batchings(4):
        seen.add(b)
        assert S.pipeline_time(4, b, 3.0, 1.0, 2.0) == HAND_N4[b], b
    assert seen == set(HAND_N4)
    t, b = S.best_batching_by_enumeration(4, 3.0, 1.0, 2.0)
    assert t == 14 and b in ((1, 2), (1, 3))


def test_three_tokens_cheap_and_dear_startup():
    # alpha = 2, beta = 1, gamma = 3: (1)=14, (1,2)=13, (1,3)=13, (1,2,3)=12 -> immediate-send wins
    vals = {b: S.pipeline_time(3, b, 2.0, 1.0, 3.0) for b in S.all_batchings(3)}
    assert vals == {(1,): 14, (1, 2): 13, (1, 3): 13, (1, 2, 3): 12}
    # alpha = 10: (1)=22, (1,2)=26, (1,3)=29, (1,2,3)=36 -> one batch wins
    vals = {b: S.pipeline_time(3, b, 10.0, 1.0, 3.0) for b in S.all_batchings(3)}
    assert vals == {(1,): 22, (1, 2): 26, (1, 3): 29, (1, 2, 3): 36}


def test_boundary_sequences_are_checked():
    for bad in ((), (2,), (1, 1), (1, 3, 2), (1, 5)):
        with pytest.raises(ValueError):
            S.pipeline_time(4, bad, 1.0, 1.0, 1.0)
    assert sum(1 for _ in S.all_batchings(7)) == 2 ** 6
    for b in S.all_batchings(6):
        assert sum(S.batch_sizes(6, b)) == 6


# ---- closed forms -----------------------------------------------------------------------------
@pytest.mark.parametrize("n", [1, 2, 5, 9])
def test_closed_forms(n):
    a, b, g = 0.75, 0.125, 0.5  # exact in binary: equalities below are exact
    # one batch: everything is generated, then sent once
    assert S.pipeline_time(n, S.no_early_upload(n), a, b, g) == g * n + a + b * n
    # no generation time: the link is the only resource, T = K alpha + beta N
    for bb in S.all_batchings(min(n, 6)):
        m = min(n, 6)
        assert S.pipeline_time(m, bb, a, b, 0.0) == len(bb) * a + b * m
    # immediate-send with alpha + beta <= gamma never queues: the last token leaves when it is ready
    assert S.pipeline_time(n, S.immediate_send(n), 0.25, 0.125, 0.5) == 0.5 * n + 0.25 + 0.125
    # immediate-send with alpha + beta >= gamma: the link is busy from the first token on
    assert S.pipeline_time(n, S.immediate_send(n), 1.0, 0.5, 0.25) == 0.25 + n * 1.5


def test_bounds_that_hold_for_every_batching():
    rng = np.random.default_rng(11)
    for _ in range(40):
        n = int(rng.integers(1, 9))
        a, b, g = (float(x) for x in rng.uniform(0.0, 3.0, 3))
        for bb in S.all_batchings(n):
            t = S.pipeline_time(n, bb, a, b, g)
            sizes = S.batch_sizes(n, bb)
            # the last batch cannot leave before the last token exists
            assert t >= g * n + a + b * sizes[-1] - 1e-12
            # nothing leaves before the first batch exists, and the link carries everything
            assert t >= g * sizes[0] + len(bb) * a + b * n - 1e-12
            # and no batching is slower than doing the two things one after the other
            assert t <= g * n + len(bb) * a + b * n + 1e-12


# ---- Theorem 1: recurrence (7) reaches the enumeration's minimum ---------------------------------
def _opt_by_recurrence(n, a, b, g):
    @functools.lru_cache(maxsize=None)
    def opt(j):
        if j == 0:
            return 0.0
        return min(max(opt(i), g * j) + a + b * (j - i) for i in range(j))
    return opt(n)


def test_enumeration_minimum_equals_recurrence_7():
    rng = np.random.default_rng(5)
    for trial in range(60):
        n = int(rng.integers(1, 11))
        if trial % 2:  # dyadic parameters: every sum is exact, so the two minima are EQUAL
            a, b, g = (float(x) / 8.0 for x in rng.integers(0, 40, 3))
            assert S.best_batching_by_enumeration(n, a, b, g)[0] == _opt_by_recurrence(n, a, b, g)
        else:
            a, b, g = (float(x) for x in rng.uniform(0.0, 5.0, 3))
            assert math.isclose(S.best_batching_by_enumeration(n, a, b, g)[0], _opt_by_recurrence(n, a, b, g),
                                rel_tol=1e-13, abs_tol=1e-13)


# ---- the alternative policies -------------------------------------------------------------------
def test_greedy_policy_by_hand():
    # N = 4, alpha = 3, beta = 1, gamma = 2: token 1 at t = 2 -> {1} on the link until 6; by then tokens
    # 2, 3 exist -> {2,3} until 11; token 4 (ready at 8) -> {4} until 15
    assert S.greedy_send(4, 3.0, 1.0, 2.0) == (1, 2, 4)
    assert S.pipeline_time(4, (1, 2, 4), 3.0, 1.0, 2.0) == 15
    # a link that is always faster than generation sends every token alone
    assert S.greedy_send(5, 0.25, 0.25, 1.0) == S.immediate_send(5)
    # no generation time: everything exists at once -> one batch
    assert S.greedy_send(5, 1.0, 1.0, 0.0) == (1,)


def test_no_policy_beats_the_optimum():
    rng = np.random.default_rng(23)
    for _ in range(50):
        n = int(rng.integers(1, 10))
        a, b, g = (float(x) for x in rng.uniform(0.0, 4.0, 3))
        t_opt, _ = S.best_batching_by_enumeration(n, a, b, g)
        for pol in (S.immediate_send(n), S.no_early_upload(n), S.greedy_send(n, a, b, g)):
            assert S.pipeline_time(n, pol, a, b, g) >= t_opt


# ---- Sec. 3.3: dual-threshold trigger -----------------------------------------------------------
def test_trigger_by_hand():
    # R1 = 0.5, R2 = 0.35.  0.9, 0.81, 0.405 <= R1 -> round of 3; 0.95, then 0.3 <= R2 -> round of 2;
    # 0.8, 0.64, 0.512, 0.4096 <= R1 -> round of 4; the trailing 0.9 triggers nothing
    conf = [0.9, 0.9, 0.5, 0.95, 0.3, 0.8, 0.8, 0.8, 0.8, 0.9]
    assert S.trigger_rounds(conf, 0.5, 0.35, 16) == [3, 2, 4]
    # the single-token threshold alone (R1 = 0 never fires for positive confidences)
    assert S.trigger_rounds(conf, 0.0, 0.5, 16) == [3, 2]
    # R1 = 1: every token fires (C1* = p <= 1)
    assert S.trigger_rounds(conf, 1.0, 0.0, 16) == [1] * len(conf)
    # neither threshold: only the length cap ends rounds
    assert S.trigger_rounds([0.99] * 10, 0.0, 0.0, 4) == [4, 4]
    assert S.trigger_rounds([], 0.5, 0.5, 4) == []


@pytest.mark.parametrize("p,r1", [(0.9, 0.5), (0.8, 0.3), (0.97, 0.6), (0.5, 0.5)])
def test_constant_confidence_gives_the_geometric_length(p, r1):
    # C1 after n tokens is p^n: the round ends at the smallest n with p^n <= R1
    n = 1
    while p ** n > r1:
        n += 1
    assert n == max(1, math.ceil(math.log(r1) / math.log(p) - 1e-12))
    rounds = S.trigger_rounds([p] * (5 * n + n - 1), r1, 0.0, 1000)  # the last n - 1 tokens fire nothing
    assert rounds == [n] * 5


def test_trigger_rounds_partition_a_prefix_of_the_stream():
    rng = np.random.default_rng(3)
    conf = rng.beta(6.0, 1.2, 500)
    for r1, r2, cap in [(0.5, 0.3, 16), (0.2, 0.6, 8), (0.9, 0.1, 31)]:
        rounds = S.trigger_rounds(conf, r1, r2, cap)
        assert all(1 <= k <= cap for k in rounds) and sum(rounds) <= len(conf)
        pos = 0
        for k in rounds:  # inside a round nothing fired before its last token; its last token fired
            seg = conf[pos:pos + k]
            c = np.cumprod(seg)
            assert np.all(c[:-1] > r1) and np.all(seg[:-1] > r2)
            assert c[-1] <= r1 or seg[-1] <= r2 or k == cap
            pos += k
