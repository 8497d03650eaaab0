"""Shared pieces of the GPU parity tests: build both sides from the same seeded inputs."""
import numpy as np

from oracle.nav import OracleSeq
from oracle.transformer import OracleModel
from paper_2605_13319_amd import inputs as I


def oracle_side(shape, weights, prefix_tokens, max_len, kv_format="model"):
    om = OracleModel(shape, weights, kv_format=kv_format)
    seq = OracleSeq(om, max_len)
    seq.prefill(prefix_tokens)
    return seq


def drafts_from_oracle(oseq, k, sigma, seed_noise, seed_u):
    """Noisy-target draft stand-in driven by the checker's logits (never by the GPU's)."""
    def logits_after(d):
        return oseq.forward_logits(d)[-1]
    return I.make_noisy_target_drafts(logits_after, k, oseq.model.s.vocab, sigma, seed_noise, seed_u)


def decision_excused(p_rows, q, drafts, u, a_gpu, a_ref, tol=1e-3):
    """End-to-end rule: an accepted-length mismatch is allowed only if the first position where the
    two sides differ has |p/q - u| < tol on the checker's probabilities."""
    i = min(a_gpu, a_ref)
    if i >= len(drafts):
        return False
    ratio = float(p_rows[i, drafts[i]]) / float(q[i, drafts[i]])
    return abs(min(1.0, ratio) - float(u[i])) < tol
