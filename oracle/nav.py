"""One sequence's state across speculative rounds on the cloud side (checker).

State between rounds: the committed tokens t_0..t_{n-1}; K/V cached for t_0..t_{n-2}; the
last committed token is pending (it was produced by the previous round's correction or extra
token, Sec. 2.2 / Appendix B, and has not been through the model yet).  Every pass therefore
runs k + 1 rows: [pending, d_1..d_k].
"""
from __future__ import annotations

import numpy as np

from .spec_sampling import greedy_accept, spec_accept
from .transformer import F32, OracleModel, softmax_rows


class OracleSeq:
    def __init__(self, model: OracleModel, max_len: int):
        s = model.s
        self.model = model
        self.K = [np.zeros((max_len, s.n_kv_heads, s.head_dim), dtype=F32) for _ in range(s.n_layers)]
        self.V = [np.zeros((max_len, s.n_kv_heads, s.head_dim), dtype=F32) for _ in range(s.n_layers)]
        self.committed: list = []
        self.cached = 0

    @property
    def prefix_len(self) -> int:
        return len(self.committed)

    def prefill(self, tokens, chunk: int = 256) -> None:
        """Commit `tokens`; cache all but the last, which stays pending."""
        assert not self.committed and len(tokens) >= 1
        self.committed = [int(t) for t in tokens]
        body = self.committed[:-1]
        for i in range(0, len(body), chunk):
            self.model.forward_rows(body[i:i + chunk], i, self.K, self.V)
        self.cached = len(body)

    def forward_logits(self, drafts) -> np.ndarray:
        """Logits of rows [pending, d_1..d_k]; leaves k + 1 uncommitted rows in the cache."""
        rows = [self.committed[-1]] + [int(t) for t in drafts]
        return self.model.forward_rows(rows, self.cached, self.K, self.V)

    def nav_verify(self, drafts, q, u) -> tuple:
        """One NAV pass + decision + rollback.  q = None selects token matching."""
        k = len(drafts)
        lp = self.prefix_len
        z = self.forward_logits(drafts)
        if q is None:
            a, nxt = greedy_accept(z, drafts)
        else:
            a, nxt = spec_accept(softmax_rows(z), q, drafts, u)
        # keep the pending row and the a accepted drafts; cut the k - a rejected rows
        self.cached = lp + a
        self.committed += [int(t) for t in drafts[:a]] + [nxt]
        return a, nxt

    def nav_verify_chain(self, rounds) -> list:
        """Proactively sent drafts (Appendix B).  rounds[0] = (drafts, q, u) is an ordinary round.
        rounds[r], r >= 1 = (buffer, q, u): `buffer` holds the tokens the edge went on drafting while
        round r - 1 was being verified, buffer[0] being its guess of that round's extra token.  The
        buffer stays valid iff every draft of round r - 1 was accepted and the extra token the
        target produced equals buffer[0]; then buffer[1:] are round r's drafts (q, u belong to
        them), otherwise this buffer and all later ones are discarded.  Returns the (accepted,
        next token) pairs of the rounds that ran."""
        out = []
        for r, (toks, q, u) in enumerate(rounds):
            toks = [int(t) for t in toks]
            if r > 0:
                a_prev, next_prev = out[-1]
                k_prev = len(rounds[r - 1][0]) - (1 if r - 1 > 0 else 0)
                if a_prev != k_prev or next_prev != toks[0]:
                    break
                toks = toks[1:]
            out.append(self.nav_verify(toks, q, u))
        return out

    def rollback(self, new_prefix_len: int) -> None:
        """Cut the committed text to `new_prefix_len` tokens; its last token becomes pending."""
        assert 1 <= new_prefix_len <= self.prefix_len
        self.committed = self.committed[:new_prefix_len]
        self.cached = new_prefix_len - 1
