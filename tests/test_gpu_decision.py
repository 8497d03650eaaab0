"""GPU parity of the decision step alone: accepted length and token index must be bit-exact with the
checker on identical fp32 probabilities and uniforms."""
import numpy as np
import pytest

from oracle.spec_sampling import spec_accept as oracle_accept
from paper_2605_13319_amd import inputs as I

pytestmark = pytest.mark.gpu
F32 = np.float32


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available()
    from paper_2605_13319_amd import nav
    return nav, torch


def _run(gpu, p, q, d, u):
    nav, torch = gpu
    return nav.spec_accept(torch.from_numpy(p).cuda(), torch.from_numpy(q).cuda(), d, u)


@pytest.mark.parametrize("V,k,scale", [(13, 1, 1.0), (16, 2, 2.0), (97, 5, 1.0), (4096, 4, 2.0), (4097, 7, 1.0),
                                       (32000, 8, 1.0), (128256, 8, 1.0), (128256, 16, 3.0), (128256, 31, 0.5),
                                       (200001, 3, 1.0)])
def test_bit_exact_random(gpu, V, k, scale):
    for trial in range(6):
        seed = 1000 * k + 17 * trial + V % 1000
        p = I.make_random_probs(k + 1, V, seed, scale)
        # drafts close to the target so that several are accepted
        q = I.make_random_probs(k, V, seed + 1, scale)
        if trial % 2 == 0:
            q = (0.8 * p[:k] + 0.2 * q).astype(F32)
        rng = np.random.default_rng(seed + 2)
        d = np.array([rng.choice(V, p=q[i].astype(np.float64) / q[i].astype(np.float64).sum()) for i in range(k)],
                     dtype=np.int32)
        u = I.make_uniforms(k + 1, seed + 3)
        print(f"case V={V} k={k} trial={trial}", flush=True)
        assert _run(gpu, p, q, d, u) == oracle_accept(p, q, d, u)


def test_bit_exact_sweep_of_the_draw(gpu):
    """One residual row, many uniforms including both ends of the range."""
    V, k = 50021, 2
    p = I.make_random_probs(k + 1, V, 5, 2.0)
    q = I.make_random_probs(k, V, 6, 2.0)
    d = np.array([int(np.argmax(q[0] / np.maximum(p[0], 1e-30))), 0], dtype=np.int32)
    us = [0.0, 2.0 ** -24, 0.25, 0.5, 0.75, 1 - 2.0 ** -24] + list(I.make_uniforms(40, 7))
    for us_ in us:
        u = np.array([1 - 2.0 ** -24, 0.5, us_], dtype=F32)
        assert _run(gpu, p, q, d, u) == oracle_accept(p, q, d, u)
    for us_ in us[:12]:
        u = np.array([0.0, 0.0, us_], dtype=F32)   # accept everything (ratios > 0): extra-token row
        assert _run(gpu, p, q, d, u) == oracle_accept(p, q, d, u)


def test_special_rows(gpu):
    V = 1000
    p = I.make_random_probs(3, V, 11)
    # q == p: all accepted
    u = I.make_uniforms(3, 12)
    d = np.array([5, 900], dtype=np.int32)
    assert _run(gpu, p, p[:2].copy(), d, u) == oracle_accept(p, p[:2].copy(), d, u)
    assert _run(gpu, p, p[:2].copy(), d, u)[0] == 2
    # draft outside the target's support: p(d) = 0 -> rejected, residual == p
    p2 = p.copy()
    p2[0, 7] = 0.0
    q = np.zeros((2, V), dtype=F32)
    q[:, 7] = 1.0
    d = np.array([7, 7], dtype=np.int32)
    assert _run(gpu, p2, q, d, u) == oracle_accept(p2, q, d, u)
    assert _run(gpu, p2, q, d, u)[0] == 0
    # q(d) = 0 < p(d): ratio = +inf accepts; p(d) = q(d) = 0 rejects
    q3 = p[:2].copy()
    q3[0, 5] = 0.0
    d = np.array([5, 900], dtype=np.int32)
    u3 = np.array([1 - 2.0 ** -24, 0.3, 0.4], dtype=F32)
    assert _run(gpu, p, q3, d, u3) == oracle_accept(p, q3, d, u3)
    p4 = p.copy()
    p4[0, 5] = 0.0
    assert _run(gpu, p4, q3, d, u3) == oracle_accept(p4, q3, d, u3)
    assert _run(gpu, p4, q3, d, u3)[0] == 0
    # residual that truncates to zero everywhere: fall back to the lowest-index maximum of p
    p5 = np.full((2, V), 1.0 / V, dtype=F32)
    p5[0, 300] = p5[0, 301] = 2.0 / V
    q5 = (p5[:1] + F32(2.0 ** -45)).astype(F32)
    q5[0, 9] = 1.0  # d = 9 is rejected for u close to 1
    d = np.array([9], dtype=np.int32)
    u5 = np.array([0.9, 0.5], dtype=F32)
    got = _run(gpu, p5, q5, d, u5)
    assert got == oracle_accept(p5, q5, d, u5)


def test_one_hot_rows_reduce_to_token_matching(gpu):
    V, k = 777, 6
    rng = np.random.default_rng(3)
    am = rng.integers(0, V, k + 1)
    p = np.zeros((k + 1, V), dtype=F32)
    p[np.arange(k + 1), am] = 1
    for cut in range(k + 1):
        d = am[:k].astype(np.int32).copy()
        if cut < k:
            d[cut] = (d[cut] + 1) % V
        q = np.zeros((k, V), dtype=F32)
        q[np.arange(k), d] = 1
        u = I.make_uniforms(k + 1, 20 + cut)
        assert _run(gpu, p, q, d, u) == (cut, int(am[cut]))
