"""The decision entry point that allocates nothing (pipesd_spec_accept_static: scratch in a static
device array) against the allocating one (pipesd_spec_accept) and the checker: bit-exact accepted
length and token index, on two calls in a row, the second on a smaller input, then a third that
reuses the scratch after both."""
import numpy as np
import pytest

from oracle.spec_sampling import spec_accept as oracle_accept
from paper_2605_13319_amd import inputs as I

pytestmark = pytest.mark.gpu
F32 = np.float32


def _case(V, k, seed):
    p = I.make_random_probs(k + 1, V, seed, 1.5)
    q = (0.7 * p[:k] + 0.3 * I.make_random_probs(k, V, seed + 1, 1.5)).astype(F32)
    rng = np.random.default_rng(seed + 2)
    d = np.array([rng.choice(V, p=q[i].astype(np.float64) / q[i].astype(np.float64).sum()) for i in range(k)],
                 dtype=np.int32)
    u = I.make_uniforms(k + 1, seed + 3)
    return p, q, d, u


def test_static_scratch_decision_equals_allocating_one():
    import torch
    assert torch.cuda.is_available()
    from paper_2605_13319_amd import nav
    out = torch.full((2,), -7, dtype=torch.int32, device="cuda")
    for V, k, seed in [(128256, 16, 11), (4099, 3, 12), (32000, 31, 13)]:  # large, then smaller, then the longest draft
        p, q, d, u = _case(V, k, seed)
        tp, tq = torch.from_numpy(p).cuda(), torch.from_numpy(q).cuda()
        print(f"case V={V} k={k} seed={seed}", flush=True)
        ref = nav.spec_accept(tp, tq, d, u)
        out.fill_(-7)
        nav.spec_accept_static(tp, tq, d, u, out)
        torch.cuda.synchronize()
        got = tuple(int(x) for x in out.cpu())
        assert got == ref, (got, ref)
        assert got == oracle_accept(p, q, d, u)


def test_static_scratch_limits_are_errors():
    import torch
    from paper_2605_13319_amd import nav
    p, q, d, u = _case(64, 2, 5)
    tp, tq = torch.from_numpy(p).cuda(), torch.from_numpy(q).cuda()
    out = torch.zeros(2, dtype=torch.int32, device="cuda")
    with pytest.raises(nav.PipesdError) as e:  # more drafts than one pass carries
        nav.spec_accept_static(torch.zeros(34, 64, device="cuda"), torch.zeros(33, 64, device="cuda"),
                               np.zeros(33, np.int32), np.zeros(34, F32), out)
    assert e.value.status == nav.EINVAL
    with pytest.raises(nav.PipesdError) as e:  # a draft token outside the vocabulary
        nav.spec_accept_static(tp, tq, np.array([1, 64], np.int32), u, out)
    assert e.value.status == nav.EINVAL
