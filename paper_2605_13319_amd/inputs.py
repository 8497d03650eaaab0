"""Seeded synthetic inputs for the NAV (non-autoregressive verification) pass.

This module only *draws* data: model shapes, random weights, token ids, noise
and uniforms.  It holds none of the method's arithmetic (no transformer forward,
no accept/reject rule), so the CPU checker and the HIP path can both be fed from
it without sharing any computation.

The paper (Sec. 2.2, Sec. 4.2) runs a decoder-only target model in the cloud but
does not say which; the shapes below are Llama-style stand-ins for the trained
model pairs of Sec. 5.1 (DeepSeek-Coder-6.7B, Llama-2-7B), with seeded random
weights and uniform-random token ids in place of HumanEval / GSM8K prompts.
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor
from typing import Callable, Dict, List, Optional, Tuple

import numpy as np

DTYPE_F32 = 0
DTYPE_BF16 = 1


@dataclasses.dataclass(frozen=True)
class ModelShape:
    """Decoder-only transformer shape (RMSNorm, rotary positions, GQA, SwiGLU FFN)."""

    name: str
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    dtype: int = DTYPE_BF16
    rms_eps: float = 1e-5
    rope_base: float = 10000.0

    def truncated(self, n_layers: int) -> "ModelShape":
        """Same width, vocab and heads with fewer layers (keeps every per-layer shape)."""
        return dataclasses.replace(self, n_layers=n_layers, name=f"{self.name}-L{n_layers}")

    @property
    def q_dim(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim

    def n_params_streamed(self) -> int:
        """Matrix elements one pass must read: all layer matrices plus the LM head."""
        per_layer = (self.q_dim + 2 * self.kv_dim) * self.d_model + self.d_model * self.q_dim \
            + 3 * self.d_ffn * self.d_model
        return self.n_layers * per_layer + self.vocab * self.d_model

    def kv_bytes_per_token(self) -> int:
        esz = 4 if self.dtype == DTYPE_F32 else 2
        return self.n_layers * 2 * self.kv_dim * esz

    def algorithmic_bytes(self, prefix_len: int, k: int, with_draft_probs: bool = True) -> int:
        """HBM bytes a pass cannot avoid: weights once, norm gains, m embedding rows,
        KV read of prefix_len + k tokens, KV write of k + 1 tokens, and the draft
        distributions (k rows of fp32)."""
        esz = 4 if self.dtype == DTYPE_F32 else 2
        m = k + 1
        w = self.n_params_streamed() * esz
        gains = (2 * self.n_layers + 1) * self.d_model * 4
        emb = m * self.d_model * esz
        kv_r = (prefix_len + k) * self.kv_bytes_per_token()
        kv_w = m * self.kv_bytes_per_token()
        q = k * self.vocab * 4 if with_draft_probs else 0
        return w + gains + emb + kv_r + kv_w + q


# The five workloads; prefix / k / noise are carried beside the shape.
TINY = ModelShape("tiny-fp32", 2, 256, 4, 4, 64, 1024, 4096, dtype=DTYPE_F32)
LLAMA_1B = ModelShape("llama-1b", 16, 2048, 32, 8, 64, 8192, 32000)
LLAMA_8B = ModelShape("llama-8b", 32, 4096, 32, 8, 128, 14336, 128256, rope_base=500000.0)
LLAMA_13B = ModelShape("llama-13b", 40, 5120, 40, 40, 128, 13824, 32000)

WORKLOADS = {
    "tiny":      dict(shape=TINY, prefix=128, k=4, sigma=None, seed=1000),
    "llama-1b":  dict(shape=LLAMA_1B, prefix=1024, k=8, sigma=0.5, seed=2000),
    "llama-8b":  dict(shape=LLAMA_8B, prefix=2048, k=8, sigma=0.5, seed=3000),
    "llama-13b": dict(shape=LLAMA_13B, prefix=8192, k=16, sigma=1.0, seed=5000),
}

# seed offsets (added to the workload's base seed)
SEED_WEIGHTS, SEED_PREFIX, SEED_NOISE, SEED_DRAFT_U, SEED_VERIFY_U, SEED_LENGTHS = 1, 2, 3, 4, 5, 6


# ----------------------------------------------------------------------------------------
# bf16 storage format (round-to-nearest-even of the fp32 bit pattern); a data format, not
# arithmetic of the method
# ----------------------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


# ----------------------------------------------------------------------------------------
# weights
# ----------------------------------------------------------------------------------------
_MATRIX_IDS = {"tok_emb": 0, "lm_head": 1, "wq": 2, "wk": 3, "wv": 4, "wo": 5,
               "w_gate": 6, "w_up": 7, "w_down": 8}


def _matrix_shapes(s: ModelShape) -> Dict[str, Tuple[int, int]]:
    return {"wq": (s.q_dim, s.d_model), "wk": (s.kv_dim, s.d_model), "wv": (s.kv_dim, s.d_model),
            "wo": (s.d_model, s.q_dim), "w_gate": (s.d_ffn, s.d_model), "w_up": (s.d_ffn, s.d_model),
            "w_down": (s.d_model, s.d_ffn)}


def _draw_matrix(seed: int, mid: int, layer: int, shape: Tuple[int, int], dtype: int, std: float):
    rng = np.random.default_rng([seed, mid, layer])
    w = rng.standard_normal(shape, dtype=np.float32)
    w *= np.float32(std)
    return f32_to_bf16_bits(w) if dtype == DTYPE_BF16 else w


def make_weights(shape: ModelShape, seed: int, std: float = 0.02, threads: int = 8) -> Dict[str, object]:
    """Every matrix ~ N(0, std^2) independently, [out][in] row-major; untied LM head; norm
    gains are 1.  fp32 shapes give float32 arrays; bf16 shapes give uint16 arrays holding
    the bf16 bit patterns of the rounded draws.  Per-layer entries are lists."""
    jobs = [("tok_emb", 0, (shape.vocab, shape.d_model)), ("lm_head", 0, (shape.vocab, shape.d_model))]
    for name, shp in _matrix_shapes(shape).items():
        for l in range(shape.n_layers):
            jobs.append((name, l, shp))
    with ThreadPoolExecutor(max_workers=max(1, threads)) as ex:
        mats = list(ex.map(lambda j: _draw_matrix(seed, _MATRIX_IDS[j[0]], j[1], j[2], shape.dtype, std), jobs))
    out: Dict[str, object] = {}
    for (name, l, _), m in zip(jobs, mats):
        if name in ("tok_emb", "lm_head"):
            out[name] = m
        else:
            out.setdefault(name, []).append(m)
    ones = np.ones(shape.d_model, dtype=np.float32)
    out["attn_norm"] = [ones.copy() for _ in range(shape.n_layers)]
    out["ffn_norm"] = [ones.copy() for _ in range(shape.n_layers)]
    out["final_norm"] = ones.copy()
    return out


# ----------------------------------------------------------------------------------------
# tokens, uniforms, noise
# ----------------------------------------------------------------------------------------
def make_tokens(n: int, vocab: int, seed: int) -> np.ndarray:
    return np.random.default_rng(seed).integers(0, vocab, size=n, dtype=np.int64).astype(np.int32)


def make_uniforms(n: int, seed: int) -> np.ndarray:
    """fp32 uniforms in [0, 1) that are exact multiples of 2^-24."""
    r = np.random.default_rng(seed).integers(0, 1 << 32, size=n, dtype=np.uint64)
    return ((r >> np.uint64(8)).astype(np.float64) * 2.0 ** -24).astype(np.float32)


def make_noise(rows: int, vocab: int, seed: int) -> np.ndarray:
    return np.random.default_rng(seed).standard_normal((rows, vocab), dtype=np.float32)


def _softmax_rows_f32(z: np.ndarray) -> np.ndarray:
    z = z.astype(np.float32)
    e = np.exp(z - z.max(axis=-1, keepdims=True))
    return (e / e.sum(axis=-1, keepdims=True, dtype=np.float32)).astype(np.float32)


def _draw_from(q: np.ndarray, u: float) -> int:
    c = np.cumsum(q.astype(np.float64))
    return int(min(np.searchsorted(c, u * c[-1], side="right"), q.shape[0] - 1))


def make_independent_drafts(k: int, vocab: int, seed_noise: int, seed_u: int, scale: float = 2.0):
    """Draft model stand-in that ignores the target: q_i = softmax(scale * N(0,1)^V),
    d_i drawn from q_i.  Returns (draft_tokens int32 [k], draft_probs fp32 [k][V])."""
    q = _softmax_rows_f32(np.float32(scale) * make_noise(k, vocab, seed_noise))
    u = make_uniforms(k, seed_u)
    d = np.array([_draw_from(q[i], float(u[i])) for i in range(k)], dtype=np.int32)
    return d, q


def make_noisy_target_drafts(target_logits_after: Callable[[List[int]], np.ndarray], k: int, vocab: int,
                             sigma: float, seed_noise: int, seed_u: int):
    """Draft model stand-in that imitates the target: for i = 1..k,
    q_i = softmax(z_i + sigma * N(0,1)^V) where z_i are the target's logits for the position
    of draft i given the committed text plus d_1..d_{i-1}, and d_i is drawn from q_i.

    `target_logits_after(drafts_so_far)` is supplied by the caller (whichever implementation
    is being fed) and must return that fp32 logit row [V] without changing persistent state."""
    noise = make_noise(k, vocab, seed_noise)
    u = make_uniforms(k, seed_u)
    d: List[int] = []
    q = np.empty((k, vocab), dtype=np.float32)
    for i in range(k):
        z = np.asarray(target_logits_after(list(d)), dtype=np.float32)
        q[i] = _softmax_rows_f32((z + np.float32(sigma) * noise[i])[None, :])[0]
        d.append(_draw_from(q[i], float(u[i])))
    return np.array(d, dtype=np.int32), q


def make_confidences(n: int, seed: int, a: float = 8.0, b: float = 1.0) -> np.ndarray:
    """Stand-in for the draft model's per-token confidences P(D_n): n draws of Beta(a, b), fp64.
    With Beta(8, 1), a single-token threshold R2 = 0.3 and a cap of 16 tokens, the dual-threshold
    trigger of Sec. 3.3 cuts the stream into rounds of mean length 6.5 at R1 = 0.5, 5.1 at R1 = 0.6
    and 4.4 at R1 = 0.65 (the paper's Table 7 reports mean draft lengths of 3.2 to 5.0)."""
    return np.random.default_rng(seed).beta(a, b, n)


def make_random_probs(rows: int, vocab: int, seed: int, scale: float = 1.0) -> np.ndarray:
    """Rows of a generic categorical distribution, fp32, for feeding the decision step alone."""
    return _softmax_rows_f32(np.float32(scale) * make_noise(rows, vocab, seed))
