"""Accept / correct / extra-token decision of one speculative round (checker).

Sec. 2.2: drafts that match what the target would generate are accepted and the first
mismatch is corrected by the target; Sec. 1: the target's output distribution is preserved
exactly; Appendix B: when every draft is accepted the target contributes one extra token.
The stochastic rule that achieves this is the speculative-sampling rule of the works cited
there: accept d_i iff u_i < min(1, p_i(d_i) / q_i(d_i)); at the first rejection draw from
max(0, p - q) normalised; after k acceptances draw the extra token from p_{k+1}.

The categorical draw uses an integer CDF so that its result does not depend on summation
order: weights are truncated to multiples of 2^-40, summed as integers, and the threshold is
floor(u * 2^24) * W / 2^24 in integer arithmetic.
"""
from __future__ import annotations

import numpy as np

F32 = np.float32
FIX_SHIFT = 40
U_BITS = 24


def draw_index(w: np.ndarray, u, fallback_row: np.ndarray) -> int:
    """Smallest j with sum_{t<=j} wi_t > T, wi = floor(w * 2^40), T = floor(u*2^24) * W >> 24.
    If every weight truncates to 0 the draw falls back to the lowest-index maximum of
    `fallback_row`."""
    wi = (w.astype(np.float64) * float(1 << FIX_SHIFT)).astype(np.uint64)
    cum = np.cumsum(wi, dtype=np.uint64)
    W = int(cum[-1])
    if W == 0:
        return int(np.argmax(fallback_row))
    u_int = int(np.float64(u) * float(1 << U_BITS))
    T = (u_int * W) >> U_BITS
    return int(np.searchsorted(cum, np.uint64(T), side="right"))


def accept_test(p: F32, q: F32, u: F32) -> bool:
    """u < min(1, p / q) with an fp32 round-to-nearest division.  q = 0 < p gives +inf, hence
    acceptance; p = q = 0 (0/0) rejects."""
    p, q, u = F32(p), F32(q), F32(u)
    if q == 0 and p == 0:
        return False
    with np.errstate(divide="ignore"):
        ratio = F32(p / q)
    return bool(u < min(F32(1.0), ratio))


def spec_accept(p: np.ndarray, q: np.ndarray, drafts, u) -> tuple:
    """p [k+1][V] target rows (row i-1 judges draft i, row k is the extra-token row),
    q [k][V] draft rows, drafts [k], u [k+1] (k tests, then one draw).
    Returns (accepted_len, next_token)."""
    k = len(drafts)
    a = 0
    while a < k and accept_test(p[a, drafts[a]], q[a, drafts[a]], u[a]):
        a += 1
    if a < k:
        w = np.maximum(F32(0.0), p[a].astype(F32) - q[a].astype(F32))
    else:
        w = p[k].astype(F32)
    return a, draw_index(w, u[k], p[a])


def greedy_accept(logits: np.ndarray, drafts) -> tuple:
    """Token matching (Sec. 2.2 as worded): accepted_len = longest prefix with
    d_i == argmax(logits[i-1]) (lowest index among equal maxima); next = argmax(logits[a])."""
    k = len(drafts)
    a = 0
    while a < k and int(np.argmax(logits[a])) == int(drafts[a]):
        a += 1
    return a, int(np.argmax(logits[a]))
