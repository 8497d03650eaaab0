"""Thin ctypes binding over the C-ABI library (include/pipesd.h): argument marshalling only.

Importing this module loads paper_2605_13319_amd/libpipesd.so and fails loudly if it has not been
built (run `python __graft_entry__.py`) or lacks a declared entry point.  PyTorch is used for
device memory and streams; every step of the NAV pass runs in the library's HIP kernels.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional, Sequence

import numpy as np
import torch  # first: the library must bind to the HIP runtime PyTorch has already loaded, not a second one

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpipesd.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python __graft_entry__.py` "
                      "(there is no CPU fallback for the NAV pass)")
_lib = C.CDLL(LIB_PATH)

OK, EINVAL, ENOMEM, ESTATE, EHIP = 0, -1, -2, -3, -4
MAX_ROWS = 32
PROF = dict(off=0, qkv=1, o=2, gateup=3, down=4, lmhead=5, attn=6, verify=7, all_gemm=8, layers=9)


class Config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("d_ffn", C.c_int32),
                ("vocab", C.c_int32), ("rms_eps", C.c_float), ("rope_base", C.c_float), ("dtype", C.c_int32)]


class Weights(C.Structure):
    _fields_ = [("tok_emb", C.c_void_p), ("final_norm", C.c_void_p), ("lm_head", C.c_void_p)] + \
               [(n, C.POINTER(C.c_void_p)) for n in ("attn_norm", "ffn_norm", "wq", "wk", "wv", "wo",
                                                      "w_gate", "w_up", "w_down")]


_i32p, _f32p = C.POINTER(C.c_int32), C.POINTER(C.c_float)
_SIGS = {
    "pipesd_model_create": (C.c_int, [C.POINTER(Config), C.POINTER(Weights), C.POINTER(C.c_void_p)]),
    "pipesd_model_destroy": (C.c_int, [C.c_void_p]),
    "pipesd_kv_block_bytes": (C.c_size_t, [C.c_void_p, C.c_int32]),
    "pipesd_kv_create": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_size_t, C.POINTER(C.c_void_p)]),
    "pipesd_kv_destroy": (C.c_int, [C.c_void_p]),
    "pipesd_seq_reset": (C.c_int, [C.c_void_p, C.c_int32]),
    "pipesd_prefill": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, _i32p, C.c_int32, C.c_void_p]),
    "pipesd_nav_verify": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, _i32p, C.c_int32, C.c_void_p,
                                    _f32p, _i32p, _i32p, C.c_void_p]),
    "pipesd_nav_verify_begin": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, _i32p, C.c_int32, C.c_void_p,
                                          _f32p, C.c_void_p]),
    "pipesd_nav_verify_done": (C.c_int, [C.c_void_p, _i32p]),
    "pipesd_nav_verify_end": (C.c_int, [C.c_void_p, _i32p, _i32p]),
    "pipesd_nav_verify_batch": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, _i32p, _i32p, _i32p, _i32p,
                                          C.POINTER(C.c_void_p), _f32p, _i32p, _i32p, C.c_void_p]),
    "pipesd_kv_rollback": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32]),
    "pipesd_kv_len": (C.c_int, [C.c_void_p, C.c_int32, _i32p]),
    "pipesd_kv_free_blocks": (C.c_int, [C.c_void_p, _i32p]),
    "pipesd_kv_seq_blocks": (C.c_int, [C.c_void_p, C.c_int32, _i32p]),
    "pipesd_forward_logits": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, _i32p, C.c_int32, _f32p, C.c_void_p]),
    "pipesd_spec_accept": (C.c_int, [C.c_void_p, C.c_void_p, _i32p, C.c_int32, C.c_int32, _f32p, _i32p, _i32p,
                                     C.c_void_p]),
    "pipesd_spec_accept_static": (C.c_int, [C.c_void_p, C.c_void_p, _i32p, C.c_int32, C.c_int32, _f32p, C.c_void_p,
                                            C.c_void_p]),
    "pipesd_kv_read": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, _f32p, _f32p]),
    "pipesd_nav_verify_chain": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, _i32p, _i32p,
                                          C.POINTER(C.c_void_p), _f32p, _i32p, _i32p, _i32p, C.c_void_p]),
    "pipesd_model_set_fused": (C.c_int, [C.c_void_p, C.c_int32]),
    "pipesd_model_set_wide_gemm": (C.c_int, [C.c_void_p, C.c_int32]),
    "pipesd_model_fused_launches": (C.c_int, [C.c_void_p, C.POINTER(C.c_int64)]),
    "pipesd_profile_select": (C.c_int, [C.c_void_p, C.c_int32]),
    "pipesd_profile_read": (C.c_int, [C.c_void_p, _i32p, C.POINTER(C.c_double)]),
    "pipesd_profile_read_each": (C.c_int, [C.c_void_p, C.POINTER(C.c_double), C.c_int32, _i32p]),
    "pipesd_profile_read_steps": (C.c_int, [C.c_void_p, C.POINTER(C.c_double), C.c_int32, _i32p]),
    "pipesd_batching_time": (C.c_int, [C.c_int32, _i32p, C.c_int32, C.c_double, C.c_double, C.c_double,
                                       C.POINTER(C.c_double)]),
    "pipesd_batching_optimal": (C.c_int, [C.c_int32, C.c_double, C.c_double, C.c_double, _i32p, _i32p,
                                          C.POINTER(C.c_double)]),
    "pipesd_trigger_rounds": (C.c_int, [C.POINTER(C.c_double), C.c_int64, C.c_double, C.c_double, C.c_int32, _i32p,
                                        C.c_int64, C.POINTER(C.c_int64), C.POINTER(C.c_int64)]),
    "pipesd_bo_posterior": (C.c_int, [C.POINTER(C.c_double), C.POINTER(C.c_double), C.c_int32, C.c_double, C.c_double,
                                      C.POINTER(C.c_double), C.c_int32, C.POINTER(C.c_double), C.POINTER(C.c_double)]),
    "pipesd_bo_suggest": (C.c_int, [C.POINTER(C.c_double), C.POINTER(C.c_double), C.c_int32, C.c_double, C.c_double,
                                    C.c_double, C.c_int32, C.POINTER(C.c_double), C.POINTER(C.c_double)]),
    "pipesd_strerror": (C.c_char_p, [C.c_int]),
    "pipesd_last_hip_error": (C.c_char_p, []),
}
for _name, (_res, _args) in _SIGS.items():
    _fn = getattr(_lib, _name)  # AttributeError = the library lacks a declared entry point
    _fn.restype, _fn.argtypes = _res, _args
EXPORTS = tuple(_SIGS)


class PipesdError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        detail = f" [{_lib.pipesd_last_hip_error().decode()}]" if status == EHIP else ""
        super().__init__(f"{where}: {_lib.pipesd_strerror(status).decode()} ({status}){detail}")


def _check(status: int, where: str) -> None:
    if status != OK:
        raise PipesdError(status, where)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _ptr(a: Optional[np.ndarray], typ):
    return None if a is None else a.ctypes.data_as(typ)


def _stream() -> int:
    return int(torch.cuda.current_stream().cuda_stream)


def batching_time(n_tokens: int, first: Sequence[int], alpha: float, beta: float, gamma: float) -> float:
    """T of Eq. (6) for the batching `first` (1-based first token of every batch)."""
    b = _i32(first)
    t = C.c_double()
    _check(_lib.pipesd_batching_time(n_tokens, _ptr(b, _i32p), len(b), alpha, beta, gamma, C.byref(t)),
           "pipesd_batching_time")
    return t.value


def batching_optimal(n_tokens: int, alpha: float, beta: float, gamma: float):
    """(first, T): the batching of minimal T for a window of n_tokens tokens (Algorithm 1)."""
    out = np.zeros(max(n_tokens, 1), dtype=np.int32)
    nb, t = C.c_int32(), C.c_double()
    _check(_lib.pipesd_batching_optimal(n_tokens, alpha, beta, gamma, _ptr(out, _i32p), C.byref(nb), C.byref(t)),
           "pipesd_batching_optimal")
    return tuple(int(x) for x in out[:nb.value]), t.value


def trigger_rounds(confidence, r1: float, r2: float, max_len: int, cap: Optional[int] = None):
    """(lengths, consumed): draft lengths of the rounds the dual-threshold trigger cuts the stream into."""
    c = np.ascontiguousarray(confidence, dtype=np.float64)
    cap = len(c) if cap is None else cap
    out = np.zeros(max(cap, 1), dtype=np.int32)
    nr, used = C.c_int64(), C.c_int64()
    _check(_lib.pipesd_trigger_rounds(c.ctypes.data_as(C.POINTER(C.c_double)), len(c), r1, r2, max_len,
                                      _ptr(out, _i32p), cap, C.byref(nr), C.byref(used)), "pipesd_trigger_rounds")
    return [int(x) for x in out[:nr.value]], int(used.value)


_f64p = C.POINTER(C.c_double)


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def bo_posterior(x, y, length_scale: float, noise: float, q):
    """GP posterior (mean, std) of the autotuner's surrogate at the query points q [m][2]."""
    x, y, q = _f64(x).reshape(-1, 2), _f64(y), _f64(q).reshape(-1, 2)
    mean, std = np.empty(len(q)), np.empty(len(q))
    _check(_lib.pipesd_bo_posterior(x.ctypes.data_as(_f64p), y.ctypes.data_as(_f64p), len(y), length_scale, noise,
                                    q.ctypes.data_as(_f64p), len(q), mean.ctypes.data_as(_f64p),
                                    std.ctypes.data_as(_f64p)), "pipesd_bo_posterior")
    return mean, std


def bo_suggest(x, y, length_scale: float, noise: float, xi: float, grid: int):
    """((R1, R2), EI): the thresholds the autotuner tries next, given the samples so far."""
    x, y = _f64(x).reshape(-1, 2), _f64(y)
    nxt = np.empty(2)
    ei = C.c_double()
    _check(_lib.pipesd_bo_suggest(x.ctypes.data_as(_f64p), y.ctypes.data_as(_f64p), len(y), length_scale, noise, xi,
                                  grid, nxt.ctypes.data_as(_f64p), C.byref(ei)), "pipesd_bo_suggest")
    return (float(nxt[0]), float(nxt[1])), ei.value


def config_of(shape) -> Config:
    return Config(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.d_ffn,
                  shape.vocab, shape.rms_eps, shape.rope_base, shape.dtype)


class Model:
    """Target model handle.  `weights` maps names to numpy arrays (float32, or uint16 bf16 bits) as
    produced by inputs.make_weights; None gives a shape-only handle (no GPU needed)."""

    def __init__(self, shape, weights: Optional[Dict[str, object]] = None, device: str = "cuda:0"):
        self.shape = shape
        self.handle = C.c_void_p()
        cfg = config_of(shape)
        if weights is None:
            _check(_lib.pipesd_model_create(C.byref(cfg), None, C.byref(self.handle)), "pipesd_model_create")
            return
        torch.cuda.set_device(device)
        keep = []

        def up(a: np.ndarray) -> int:
            t = torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).to(device)
            keep.append(t)
            return t.data_ptr()

        w = Weights()
        w.tok_emb, w.final_norm, w.lm_head = up(weights["tok_emb"]), up(weights["final_norm"]), up(weights["lm_head"])
        arrays = []
        for name in ("attn_norm", "ffn_norm", "wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down"):
            arr = (C.c_void_p * shape.n_layers)(*[up(a) for a in weights[name]])
            arrays.append(arr)
            setattr(w, name, arr)
        torch.cuda.synchronize()
        _check(_lib.pipesd_model_create(C.byref(cfg), C.byref(w), C.byref(self.handle)), "pipesd_model_create")
        del keep  # the library holds its own re-tiled copies

    def close(self) -> None:
        if self.handle:
            _lib.pipesd_model_destroy(self.handle)
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_wide_gemm(self, mode: int) -> None:
        """GEMM kernel of passes of more than 64 rows: 0 by shape, 1 narrow, 2 wide (same results)."""
        _check(_lib.pipesd_model_set_wide_gemm(self.handle, int(mode)), "pipesd_model_set_wide_gemm")

    def set_fused(self, on: bool) -> None:
        _check(_lib.pipesd_model_set_fused(self.handle, 1 if on else 0), "pipesd_model_set_fused")

    def fused_launches(self) -> int:
        n = C.c_int64()
        _check(_lib.pipesd_model_fused_launches(self.handle, C.byref(n)), "pipesd_model_fused_launches")
        return n.value

    def profile_select(self, which: str) -> None:
        _check(_lib.pipesd_profile_select(self.handle, PROF[which]), "pipesd_profile_select")

    def profile_read(self):
        n, ms = C.c_int32(), C.c_double()
        _check(_lib.pipesd_profile_read(self.handle, C.byref(n), C.byref(ms)), "pipesd_profile_read")
        return n.value, ms.value

    def profile_read_each(self, cap: int = 1 << 16):
        """Durations (us) of the timed launches since the last read, in launch order."""
        buf = (C.c_double * cap)()
        n = C.c_int32()
        _check(_lib.pipesd_profile_read_each(self.handle, buf, cap, C.byref(n)), "pipesd_profile_read_each")
        return [buf[i] for i in range(min(n.value, cap))]

    def profile_read_steps(self):
        """Durations (us) of the 4 * n_layers steps of the most recent fused launch."""
        cap = 4 * self.shape.n_layers
        buf = (C.c_double * cap)()
        n = C.c_int32()
        _check(_lib.pipesd_profile_read_steps(self.handle, buf, cap, C.byref(n)), "pipesd_profile_read_steps")
        return [buf[i] for i in range(min(n.value, cap))]


class KVCache:
    """Paged KV cache over a torch-allocated device pool (or bookkeeping only when the model is
    shape-only)."""

    def __init__(self, model: Model, max_seqs: int, n_blocks: int, block_tokens: int = 16,
                 device: str = "cuda:0", on_device: Optional[bool] = None):
        self.model = model
        self.handle = C.c_void_p()
        bb = _lib.pipesd_kv_block_bytes(model.handle, block_tokens)
        if bb == 0:
            raise PipesdError(EINVAL, "pipesd_kv_block_bytes")
        self.block_bytes = bb
        self.pool = None
        pool_ptr = None
        if on_device is None:
            on_device = True
        if on_device:
            self.pool = torch.zeros(n_blocks * bb, dtype=torch.uint8, device=device)
            pool_ptr = self.pool.data_ptr()
        _check(_lib.pipesd_kv_create(model.handle, max_seqs, block_tokens, pool_ptr, n_blocks * bb,
                                     C.byref(self.handle)), "pipesd_kv_create")

    def close(self) -> None:
        if self.handle:
            _lib.pipesd_kv_destroy(self.handle)
            self.handle = C.c_void_p()
            self.pool = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def reset(self, seq: int) -> None:
        _check(_lib.pipesd_seq_reset(self.handle, seq), "pipesd_seq_reset")

    def prefill(self, seq: int, tokens: Sequence[int]) -> None:
        t = _i32(tokens)
        _check(_lib.pipesd_prefill(self.model.handle, self.handle, seq, _ptr(t, _i32p), len(t), _stream()),
               "pipesd_prefill")

    def nav_verify(self, seq: int, drafts: Sequence[int], draft_probs=None, uniforms=None,
                   prefix_len: Optional[int] = None):
        """draft_probs: torch CUDA float32 tensor [k][V], or numpy (uploaded), or None (token matching)."""
        d = _i32(drafts)
        k = len(d)
        qptr, keep = None, None
        if draft_probs is not None:
            if isinstance(draft_probs, np.ndarray):
                keep = torch.from_numpy(_f32(draft_probs)).cuda()
            else:
                keep = draft_probs.contiguous()
            assert keep.dtype == torch.float32 and keep.numel() == k * self.model.shape.vocab
            qptr = keep.data_ptr()
        u = None if uniforms is None else _f32(uniforms)
        if prefix_len is None:
            prefix_len = self.length(seq)
        a, n = C.c_int32(-1), C.c_int32(-1)
        _check(_lib.pipesd_nav_verify(self.model.handle, self.handle, seq, prefix_len, _ptr(d, _i32p), k, qptr,
                                      _ptr(u, _f32p), C.byref(a), C.byref(n), _stream()), "pipesd_nav_verify")
        return a.value, n.value

    def nav_verify_begin(self, seq: int, drafts: Sequence[int], draft_probs=None, uniforms=None,
                         prefix_len: Optional[int] = None) -> None:
        """First half of nav_verify: enqueues the pass and returns without waiting.  The draft
        distributions are kept alive until nav_verify_end."""
        d = _i32(drafts)
        k = len(d)
        qptr, keep = None, None
        if draft_probs is not None:
            if isinstance(draft_probs, np.ndarray):
                keep = torch.from_numpy(_f32(draft_probs)).cuda()
            else:
                keep = draft_probs.contiguous()
            assert keep.dtype == torch.float32 and keep.numel() == k * self.model.shape.vocab
            qptr = keep.data_ptr()
        u = None if uniforms is None else _f32(uniforms)
        if prefix_len is None:
            prefix_len = self.length(seq)
        _check(_lib.pipesd_nav_verify_begin(self.model.handle, self.handle, seq, prefix_len, _ptr(d, _i32p), k, qptr,
                                            _ptr(u, _f32p), _stream()), "pipesd_nav_verify_begin")
        self._pending_keep = keep

    def nav_verify_done(self) -> bool:
        done = C.c_int32(0)
        _check(_lib.pipesd_nav_verify_done(self.model.handle, C.byref(done)), "pipesd_nav_verify_done")
        return bool(done.value)

    def nav_verify_end(self):
        """Second half of nav_verify: waits for the pass begun last and books it; (accepted_len, next_token)."""
        a, n = C.c_int32(-1), C.c_int32(-1)
        try:
            _check(_lib.pipesd_nav_verify_end(self.model.handle, C.byref(a), C.byref(n)), "pipesd_nav_verify_end")
        finally:
            self._pending_keep = None
        return a.value, n.value

    def nav_verify_batch(self, seqs: Sequence[int], drafts: Sequence[Sequence[int]], draft_probs=None,
                         uniforms=None, prefix_lens: Optional[Sequence[int]] = None):
        """One pass per client in `seqs`.  drafts[i]: the client's draft tokens; draft_probs: None, or a
        list whose entries are torch CUDA float32 tensors [k_i][V], numpy arrays (uploaded) or None;
        uniforms: list of k_i + 1 values per client (may be None for token-matching clients).
        Returns (accepted_len list, next_token list)."""
        n = len(seqs)
        ks = _i32([len(d) for d in drafts])
        cat = _i32([t for d in drafts for t in d])
        keep = []
        qarr = None
        if draft_probs is not None:
            qarr = (C.c_void_p * n)()
            for i, q in enumerate(draft_probs):
                if q is None:
                    qarr[i] = None
                    continue
                t = torch.from_numpy(_f32(q)).cuda() if isinstance(q, np.ndarray) else q.contiguous()
                assert t.dtype == torch.float32 and t.numel() == len(drafts[i]) * self.model.shape.vocab
                keep.append(t)
                qarr[i] = t.data_ptr()
        ucat = None
        if uniforms is not None:
            flat = []
            for i in range(n):
                ui = uniforms[i]
                flat.extend([0.0] * (len(drafts[i]) + 1) if ui is None else list(ui))
            ucat = _f32(flat)
        if prefix_lens is None:
            prefix_lens = [self.length(s) for s in seqs]
        ids, pl = _i32(seqs), _i32(prefix_lens)
        a = np.full(n, -1, dtype=np.int32)
        nx = np.full(n, -1, dtype=np.int32)
        _check(_lib.pipesd_nav_verify_batch(self.model.handle, self.handle, n, _ptr(ids, _i32p), _ptr(pl, _i32p),
                                            _ptr(ks, _i32p), _ptr(cat, _i32p), qarr, _ptr(ucat, _f32p),
                                            _ptr(a, _i32p), _ptr(nx, _i32p), _stream()), "pipesd_nav_verify_batch")
        return a.tolist(), nx.tolist()

    def nav_verify_chain(self, seq: int, rounds, prefix_len: Optional[int] = None):
        """Chained rounds on proactively sent drafts.  rounds[0] = (drafts, q, u); rounds[r >= 1] =
        (buffer, q, u) with buffer[0] the guess of the previous round's extra token and buffer[1:]
        the round's drafts (q: [k][V] array / CUDA tensor for the drafts, or None; u: k + 1 values or
        None).  Returns the (accepted_len, next_token) pairs of the rounds that ran."""
        n = len(rounds)
        ks = _i32([len(t) - (1 if r > 0 else 0) for r, (t, _, _) in enumerate(rounds)])
        cat = _i32([int(x) for t, _, _ in rounds for x in t])
        keep, qarr, flat, any_q = [], (C.c_void_p * n)(), [], False
        for r, (t, q, u) in enumerate(rounds):
            k = int(ks[r])
            if q is None:
                qarr[r] = None
            else:
                tq = torch.from_numpy(_f32(q)).cuda() if isinstance(q, np.ndarray) else q.contiguous()
                assert tq.dtype == torch.float32 and tq.numel() == k * self.model.shape.vocab
                keep.append(tq)
                qarr[r] = tq.data_ptr()
                any_q = True
            flat.extend([0.0] * (k + 1) if u is None else list(u))
        ucat = _f32(flat)
        if prefix_len is None:
            prefix_len = self.length(seq)
        a = np.full(n, -1, dtype=np.int32)
        nx = np.full(n, -1, dtype=np.int32)
        ran = _i32([0])
        _check(_lib.pipesd_nav_verify_chain(self.model.handle, self.handle, seq, prefix_len, n, _ptr(ks, _i32p),
                                            _ptr(cat, _i32p), qarr if any_q else None, _ptr(ucat, _f32p),
                                            _ptr(a, _i32p), _ptr(nx, _i32p), _ptr(ran, _i32p), _stream()),
               "pipesd_nav_verify_chain")
        return [(int(a[r]), int(nx[r])) for r in range(int(ran[0]))]

    def rollback(self, seq: int, new_prefix_len: int) -> None:
        _check(_lib.pipesd_kv_rollback(self.handle, seq, new_prefix_len), "pipesd_kv_rollback")

    def length(self, seq: int) -> int:
        n = C.c_int32()
        _check(_lib.pipesd_kv_len(self.handle, seq, C.byref(n)), "pipesd_kv_len")
        return n.value

    def free_blocks(self) -> int:
        n = C.c_int32()
        _check(_lib.pipesd_kv_free_blocks(self.handle, C.byref(n)), "pipesd_kv_free_blocks")
        return n.value

    def seq_blocks(self, seq: int) -> int:
        n = C.c_int32()
        _check(_lib.pipesd_kv_seq_blocks(self.handle, seq, C.byref(n)), "pipesd_kv_seq_blocks")
        return n.value

    def forward_logits(self, seq: int, tokens: Sequence[int] = ()) -> np.ndarray:
        t = _i32(tokens)
        out = np.empty((len(t) + 1, self.model.shape.vocab), dtype=np.float32)
        _check(_lib.pipesd_forward_logits(self.model.handle, self.handle, seq, _ptr(t, _i32p) if len(t) else None,
                                          len(t), _ptr(out, _f32p), _stream()), "pipesd_forward_logits")
        return out

    def read_kv(self, seq: int, layer: int, pos: int):
        s = self.model.shape
        k = np.empty(s.n_kv_heads * s.head_dim, dtype=np.float32)
        v = np.empty_like(k)
        _check(_lib.pipesd_kv_read(self.model.handle, self.handle, seq, layer, pos, _ptr(k, _f32p), _ptr(v, _f32p)),
               "pipesd_kv_read")
        return k, v


def spec_accept(p, q, drafts: Sequence[int], uniforms) -> tuple:
    """Decision step alone on device tensors p [k+1][V], q [k][V] (torch CUDA float32)."""
    d = _i32(drafts)
    u = _f32(uniforms)
    k = len(d)
    vocab = p.shape[-1]
    assert p.is_contiguous() and q.is_contiguous() and p.shape[0] == k + 1 and q.shape[0] == k
    a, n = C.c_int32(-1), C.c_int32(-1)
    _check(_lib.pipesd_spec_accept(p.data_ptr(), q.data_ptr(), _ptr(d, _i32p), k, vocab, _ptr(u, _f32p), C.byref(a),
                                   C.byref(n), _stream()), "pipesd_spec_accept")
    return a.value, n.value


def spec_accept_static(p, q, drafts: Sequence[int], uniforms, result) -> None:
    """The decision step through the entry point that allocates nothing: enqueues the work on the
    current stream and returns; `result` (torch CUDA int32 tensor of 2) holds {accepted_len,
    next_token} once the stream has been synchronised."""
    d = _i32(drafts)
    u = _f32(uniforms)
    k = len(d)
    vocab = p.shape[-1]
    assert p.is_contiguous() and q.is_contiguous() and p.shape[0] == k + 1 and q.shape[0] == k
    assert result.dtype == torch.int32 and result.numel() >= 2 and result.is_cuda
    _check(_lib.pipesd_spec_accept_static(p.data_ptr(), q.data_ptr(), _ptr(d, _i32p), k, vocab, _ptr(u, _f32p),
                                          result.data_ptr(), _stream()), "pipesd_spec_accept_static")
