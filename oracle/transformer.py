"""Decoder-only transformer forward, written out plainly (checker; see package docstring).

The paper only says the target is a decoder-only stack of masked self-attention and
feed-forward layers (Sec. 2.1); the concrete layer (RMSNorm, rotary positions on pairs
(i, i + h/2), grouped-query attention, SwiGLU, no biases, untied LM head) is the Llama-style
reading taken here (the paper evaluates Llama-family targets, Sec. 5.1).
"""
from __future__ import annotations

import numpy as np

F32 = np.float32


def widen(w) -> np.ndarray:
    """Weights arrive as float32, or as uint16 holding bf16 bit patterns (widened exactly)."""
    if w.dtype == np.uint16:
        return (w.astype(np.uint32) << np.uint32(16)).view(np.float32)
    return w


def to_cache_format(x: np.ndarray, bf16: bool) -> np.ndarray:
    """Keys and values are stored in the model's storage type.  For bf16 models that is a
    round-to-nearest-even of the fp32 value to 8 significand bits; later reads see that value."""
    if not bf16:
        return x
    b = np.ascontiguousarray(x, dtype=F32).view(np.uint32)
    r = ((b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)) << np.uint32(16)
    return r.view(F32).reshape(x.shape)


def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    """h = x / sqrt(mean(x^2) + eps) * g, per row."""
    ms = np.mean(x.astype(F32) ** 2, axis=-1, keepdims=True, dtype=F32)
    return (x * (F32(1.0) / np.sqrt(ms + F32(eps)))) * g


def rope_tables(positions: np.ndarray, head_dim: int, base: float):
    """cos/sin of pos * base^(-2i/h), i = 0..h/2-1; angles in fp64, tables rounded to fp32."""
    i = np.arange(head_dim // 2, dtype=np.float64)
    theta = np.float64(base) ** (-2.0 * i / head_dim)
    ang = positions.astype(np.float64)[:, None] * theta[None, :]
    return np.cos(ang).astype(F32), np.sin(ang).astype(F32)


def rope(v: np.ndarray, cos: np.ndarray, sin: np.ndarray) -> np.ndarray:
    """v [rows, heads, h]; element i pairs with i + h/2 and the pair is rotated by the angle."""
    half = v.shape[-1] // 2
    a, b = v[..., :half], v[..., half:]
    c, s = cos[:, None, :], sin[:, None, :]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1).astype(F32)


def softmax_rows(z: np.ndarray) -> np.ndarray:
    z = z.astype(F32)
    e = np.exp(z - np.max(z, axis=-1, keepdims=True))
    return (e / np.sum(e, axis=-1, keepdims=True, dtype=F32)).astype(F32)


def silu(t: np.ndarray) -> np.ndarray:
    return t / (F32(1.0) + np.exp(-t))


class OracleModel:
    """kv_format selects what the cache holds.  "model" (default): the model's storage type, i.e. a
    bf16 model keeps keys and values rounded to bf16 (the cache is part of the sequence's state and
    has a format).  "fp32": keys and values stay fp32 whatever the model's storage type; with it the
    checker is fp32 throughout, which is the yardstick for how far a bf16 cache moves the logits."""

    def __init__(self, shape, weights, kv_format: str = "model"):
        assert kv_format in ("model", "fp32")
        self.s = shape
        self.w = weights
        self.kv_bf16 = kv_format == "model" and shape.dtype == 1

    def forward_rows(self, tokens, start_pos: int, K: list, V: list) -> np.ndarray:
        """Rows r = 0..m-1 carry `tokens[r]` at position start_pos + r.  K[l], V[l] are
        [max_len, n_kv_heads, head_dim] fp32 arrays holding positions < start_pos; this call
        writes positions start_pos..start_pos+m-1 and returns the m x vocab fp32 logits."""
        s, w = self.s, self.w
        tokens = np.asarray(tokens, dtype=np.int64)
        m = tokens.shape[0]
        pos = start_pos + np.arange(m)
        cos, sin = rope_tables(pos, s.head_dim, s.rope_base)
        group = s.n_q_heads // s.n_kv_heads
        scale = F32(1.0 / np.sqrt(s.head_dim))
        # row r may look at key positions 0..pos_r
        allowed = np.arange(start_pos + m)[None, :] <= pos[:, None]

        x = widen(w["tok_emb"][tokens]).astype(F32)
        for l in range(s.n_layers):
            h = rmsnorm(x, w["attn_norm"][l], s.rms_eps)
            q = (h @ widen(w["wq"][l]).T).reshape(m, s.n_q_heads, s.head_dim)
            k = (h @ widen(w["wk"][l]).T).reshape(m, s.n_kv_heads, s.head_dim)
            v = (h @ widen(w["wv"][l]).T).reshape(m, s.n_kv_heads, s.head_dim)
            q = rope(q, cos, sin)
            k = rope(k, cos, sin)
            K[l][start_pos:start_pos + m] = to_cache_format(k, self.kv_bf16)
            V[l][start_pos:start_pos + m] = to_cache_format(v, self.kv_bf16)
            o = np.empty((m, s.n_q_heads, s.head_dim), dtype=F32)
            for g in range(s.n_q_heads):
                kvh = g // group
                keys = K[l][:start_pos + m, kvh, :]
                vals = V[l][:start_pos + m, kvh, :]
                sc = (q[:, g, :] @ keys.T) * scale
                sc = np.where(allowed, sc, F32(-np.inf))
                o[:, g, :] = softmax_rows(sc) @ vals
            x = x + o.reshape(m, s.q_dim) @ widen(w["wo"][l]).T
            h = rmsnorm(x, w["ffn_norm"][l], s.rms_eps)
            a = silu(h @ widen(w["w_gate"][l]).T) * (h @ widen(w["w_up"][l]).T)
            x = x + a @ widen(w["w_down"][l]).T
        return (rmsnorm(x, w["final_norm"], s.rms_eps) @ widen(w["lm_head"]).T).astype(F32)
