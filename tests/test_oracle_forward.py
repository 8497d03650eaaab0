"""Pins for the checker's transformer forward and sequence state (oracle/transformer.py,
oracle/nav.py): identities that hold by definition, a hand-computed example, and an
independent re-statement with torch primitives."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as Fn

from oracle.nav import OracleSeq
from oracle.transformer import OracleModel, rmsnorm, rope, rope_tables, softmax_rows, widen
from paper_2605_13319_amd import inputs as I

F32 = np.float32
SMALL = I.ModelShape("pin-gqa", 2, 64, 4, 2, 16, 128, 97, dtype=I.DTYPE_F32, rope_base=100.0)
SMALL_BF16 = I.ModelShape("pin-bf16", 2, 64, 4, 2, 16, 128, 97, dtype=I.DTYPE_BF16)


def _model(shape=SMALL, seed=5, std=0.25):
    w = I.make_weights(shape, seed, std=std, threads=2)
    rng = np.random.default_rng(seed + 100)
    # non-trivial gains so a dropped gain fails
    w["attn_norm"] = [(1 + 0.3 * rng.standard_normal(shape.d_model)).astype(F32) for _ in range(shape.n_layers)]
    w["ffn_norm"] = [(1 + 0.3 * rng.standard_normal(shape.d_model)).astype(F32) for _ in range(shape.n_layers)]
    w["final_norm"] = (1 + 0.3 * rng.standard_normal(shape.d_model)).astype(F32)
    return OracleModel(shape, w)


def test_row_block_equals_sequential_single_token_forwards():
    m = _model()
    toks = I.make_tokens(23, SMALL.vocab, 1)
    a = OracleSeq(m, 64)
    za = m.forward_rows(toks, 0, a.K, a.V)
    b = OracleSeq(m, 64)
    zb = np.stack([m.forward_rows(toks[i:i + 1], i, b.K, b.V)[0] for i in range(len(toks))])
    assert np.abs(za - zb).max() < 1e-5 * max(1.0, np.abs(za).max())
    # and in uneven chunks on top of a cached prefix
    c = OracleSeq(m, 64)
    zc = np.concatenate([m.forward_rows(toks[:7], 0, c.K, c.V), m.forward_rows(toks[7:12], 7, c.K, c.V),
                         m.forward_rows(toks[12:], 12, c.K, c.V)])
    assert np.abs(za - zc).max() < 1e-5 * max(1.0, np.abs(za).max())
    for l in range(SMALL.n_layers):
        np.testing.assert_allclose(a.K[l][:23], c.K[l][:23], atol=1e-5)
        np.testing.assert_allclose(a.V[l][:23], c.V[l][:23], atol=1e-5)


def test_causality_future_rows_do_not_change_earlier_logits():
    m = _model()
    toks = I.make_tokens(12, SMALL.vocab, 2)
    s1, s2 = OracleSeq(m, 32), OracleSeq(m, 32)
    z1 = m.forward_rows(toks, 0, s1.K, s1.V)
    toks2 = toks.copy()
    toks2[8:] = (toks2[8:] + 1) % SMALL.vocab
    z2 = m.forward_rows(toks2, 0, s2.K, s2.V)
    np.testing.assert_array_equal(z1[:8], z2[:8])
    assert np.abs(z1[8:] - z2[8:]).max() > 1e-3


def _torch_forward(shape, w, tokens, bf16_cache=None):
    """The same model re-stated with torch.nn.functional primitives, fp64, rotary positions
    as complex multiplication.  Shares nothing with the checker but the weights.
    bf16_cache: whether keys and values are rounded to bf16 (default: iff the model is bf16)."""
    if bf16_cache is None:
        bf16_cache = shape.dtype == I.DTYPE_BF16
    t = lambda a: torch.from_numpy(np.array(widen(a), dtype=np.float64))
    n = len(tokens)
    x = Fn.embedding(torch.as_tensor(np.asarray(tokens, dtype=np.int64)), t(w["tok_emb"]))
    half = shape.head_dim // 2
    freqs = torch.pow(torch.tensor(shape.rope_base, dtype=torch.float64),
                      -torch.arange(half, dtype=torch.float64) * 2 / shape.head_dim)
    rot = torch.polar(torch.ones(n, half, dtype=torch.float64),
                      torch.arange(n, dtype=torch.float64)[:, None] * freqs[None])

    def rotary(v):  # [n, heads, h]
        z = torch.complex(v[..., :half], v[..., half:]) * rot[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)

    rep = shape.n_q_heads // shape.n_kv_heads
    for l in range(shape.n_layers):
        h = Fn.rms_norm(x, (shape.d_model,), t(w["attn_norm"][l]), eps=shape.rms_eps)
        q = rotary(Fn.linear(h, t(w["wq"][l])).view(n, shape.n_q_heads, shape.head_dim))
        k = rotary(Fn.linear(h, t(w["wk"][l])).view(n, shape.n_kv_heads, shape.head_dim))
        v = Fn.linear(h, t(w["wv"][l])).view(n, shape.n_kv_heads, shape.head_dim)
        if bf16_cache:  # a bf16 model keeps its cache in bf16
            k = k.to(torch.float32).to(torch.bfloat16).to(torch.float64)
            v = v.to(torch.float32).to(torch.bfloat16).to(torch.float64)
        k = k.repeat_interleave(rep, dim=1)
        v = v.repeat_interleave(rep, dim=1)
        o = Fn.scaled_dot_product_attention(q.transpose(0, 1), k.transpose(0, 1), v.transpose(0, 1), is_causal=True)
        x = x + Fn.linear(o.transpose(0, 1).reshape(n, -1), t(w["wo"][l]))
        h = Fn.rms_norm(x, (shape.d_model,), t(w["ffn_norm"][l]), eps=shape.rms_eps)
        x = x + Fn.linear(Fn.silu(Fn.linear(h, t(w["w_gate"][l]))) * Fn.linear(h, t(w["w_up"][l])), t(w["w_down"][l]))
    h = Fn.rms_norm(x, (shape.d_model,), t(w["final_norm"]), eps=shape.rms_eps)
    return Fn.linear(h, t(w["lm_head"])).numpy()


@pytest.mark.parametrize("shape", [SMALL, SMALL_BF16])
def test_forward_matches_torch_restatement(shape):
    m = _model(shape)
    toks = I.make_tokens(19, shape.vocab, 3)
    s = OracleSeq(m, 32)
    z = m.forward_rows(toks, 0, s.K, s.V)
    zt = _torch_forward(shape, m.w, toks)
    assert np.abs(zt).max() > 0.5
    # bf16 cache: a key/value that sits on a rounding boundary may land one bf16 step apart in the
    # two computations (fp32 here, fp64 there), which moves logits by ~1e-4; mistakes move them by O(1)
    tol = 2e-5 if shape.dtype == I.DTYPE_F32 else 2e-4
    assert np.abs(z - zt).max() < tol * max(1.0, np.abs(zt).max())


def test_fp32_cache_switch_is_fp32_throughout():
    """kv_format="fp32" on a bf16 model: no rounding anywhere after the weights, so the checker meets
    the un-rounded fp64 restatement at the fp32 bar, and differs from its own bf16-cache run by the
    cache rounding (visible, but small on this shape)."""
    shape = SMALL_BF16
    m16 = _model(shape)
    m32 = OracleModel(shape, m16.w, kv_format="fp32")
    toks = I.make_tokens(19, shape.vocab, 3)
    s16, s32 = OracleSeq(m16, 32), OracleSeq(m32, 32)
    z16 = m16.forward_rows(toks, 0, s16.K, s16.V)
    z32 = m32.forward_rows(toks, 0, s32.K, s32.V)
    zt = _torch_forward(shape, m16.w, toks, bf16_cache=False)
    assert np.abs(z32 - zt).max() < 2e-5 * max(1.0, np.abs(zt).max())
    gap = float(np.abs(z16 - z32).max())
    assert 1e-5 < gap < 5e-2, gap
    # the cache itself: fp32 run keeps more than 8 significand bits, the bf16 run exactly 8
    k32, k16 = s32.K[0][:18].view(np.uint32), s16.K[0][:18].view(np.uint32)
    assert (k32 & 0xFFFF).any() and not (k16 & 0xFFFF).any()
    # an fp32 model ignores the switch
    mf = _model(SMALL)
    mf2 = OracleModel(SMALL, mf.w, kv_format="fp32")
    a, b = OracleSeq(mf, 32), OracleSeq(mf2, 32)
    np.testing.assert_array_equal(mf.forward_rows(toks, 0, a.K, a.V), mf2.forward_rows(toks, 0, b.K, b.V))


def test_cache_format_is_bf16_round_to_nearest_even_bit_for_bit():
    """to_cache_format against the format's definition on hand-picked patterns (ties go to the even
    8-bit significand, subnormals, infinities, the largest finite value rounding up to infinity) and
    against torch's independent float32 -> bfloat16 conversion on 10^6 random bit patterns."""
    from oracle.transformer import to_cache_format

    def bits(u):
        return np.array(u, dtype=np.uint32).view(F32)

    cases = {  # fp32 bits -> expected bf16 bits (upper half of the fp32 word)
        0x3F800000: 0x3F80,  # 1.0 exactly
        0x3F808000: 0x3F80,  # 1 + 2^-8: tie, even neighbour is 1.0
        0x3F818000: 0x3F82,  # 1 + 3*2^-8: tie, even neighbour is 1 + 2^-6
        0x3F808001: 0x3F81,  # just above the tie: up
        0x3F807FFF: 0x3F80,  # just below the tie: down
        0xBF808000: 0xBF80,  # the same tie, negative
        0xBF818000: 0xBF82,
        0x00000001: 0x0000,  # smallest fp32 subnormal -> +0
        0x00008000: 0x0000,  # subnormal tie between 0 and the smallest bf16 subnormal: even is 0
        0x00018000: 0x0002,  # subnormal tie, even neighbour above
        0x00008001: 0x0001,  # above the tie: smallest bf16 subnormal
        0x80008001: 0x8001,
        0x007F8000: 0x0080,  # largest-subnormal region tie rounds into the smallest normal
        0x7F7FFFFF: 0x7F80,  # largest finite fp32 rounds to +inf
        0x7F7F7FFF: 0x7F7F,  # just below the tie under the largest bf16
        0x7F800000: 0x7F80,  # +inf
        0xFF800000: 0xFF80,  # -inf
        0x00000000: 0x0000,
        0x80000000: 0x8000,  # -0 keeps its sign
    }
    src = bits(list(cases.keys()))
    got = to_cache_format(src, True).view(np.uint32)
    want = np.array([v << 16 for v in cases.values()], dtype=np.uint32)
    np.testing.assert_array_equal(got, want)
    np.testing.assert_array_equal(to_cache_format(src, False).view(np.uint32), src.view(np.uint32))  # fp32: untouched
    rng = np.random.default_rng(123)
    raw = rng.integers(0, 2 ** 32, 1_000_000, dtype=np.uint64).astype(np.uint32)
    raw = raw[(raw & 0x7F800000) != 0x7F800000]  # finite values and both zeros; inf covered above, NaN never cached
    x = raw.view(F32)
    ref = torch.from_numpy(x.copy()).to(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(to_cache_format(x, True).view(np.uint32), ref.view(np.uint32))
    # shape is kept
    assert to_cache_format(np.zeros((3, 2, 4), F32), True).shape == (3, 2, 4)


def test_gqa_with_repeated_kv_heads_equals_mha():
    m = _model()
    mha = I.ModelShape("pin-mha", 2, 64, 4, 4, 16, 128, 97, dtype=I.DTYPE_F32, rope_base=100.0)
    w2 = dict(m.w)
    rep = lambda a: np.repeat(a.reshape(2, 16, 64), 2, axis=0).reshape(64, 64)
    w2["wk"] = [rep(a) for a in m.w["wk"]]
    w2["wv"] = [rep(a) for a in m.w["wv"]]
    m2 = OracleModel(mha, w2)
    toks = I.make_tokens(9, 97, 4)
    s1, s2 = OracleSeq(m, 16), OracleSeq(m2, 16)
    np.testing.assert_allclose(m.forward_rows(toks, 0, s1.K, s1.V), m2.forward_rows(toks, 0, s2.K, s2.V), atol=1e-5)


def test_hand_computed_two_token_example():
    """One layer, d = 2, one head.  W_q = 0 makes attention uniform over the visible keys;
    everything else is small enough to evaluate with Python floats."""
    shp = I.ModelShape("hand", 1, 2, 1, 1, 2, 2, 3, dtype=I.DTYPE_F32, rms_eps=0.0, rope_base=10000.0)
    E = np.array([[3.0, 4.0], [1.0, 0.0], [0.0, 2.0]], dtype=F32)
    Wv = np.array([[1.0, 0.0], [1.0, 1.0]], dtype=F32)
    Wo = np.array([[2.0, 0.0], [0.0, 1.0]], dtype=F32)
    Wg = np.array([[1.0, 0.0], [0.0, 1.0]], dtype=F32)
    Wu = np.array([[0.0, 1.0], [1.0, 0.0]], dtype=F32)
    Wd = np.array([[1.0, 1.0], [0.0, 1.0]], dtype=F32)
    LM = np.array([[1.0, 0.0], [0.0, 1.0], [1.0, -1.0]], dtype=F32)
    w = dict(tok_emb=E, lm_head=LM, wq=[np.zeros((2, 2), F32)], wk=[np.eye(2, dtype=F32)], wv=[Wv], wo=[Wo],
             w_gate=[Wg], w_up=[Wu], w_down=[Wd], attn_norm=[np.ones(2, F32)], ffn_norm=[np.array([2.0, 1.0], F32)],
             final_norm=np.ones(2, F32))
    m = OracleModel(shp, w)
    s = OracleSeq(m, 4)
    z = m.forward_rows([0, 1], 0, s.K, s.V)

    def norm(v, g=(1.0, 1.0)):
        r = math.sqrt((v[0] ** 2 + v[1] ** 2) / 2)
        return [v[0] / r * g[0], v[1] / r * g[1]]

    def mv(W, v):
        return [float(W[i][0]) * v[0] + float(W[i][1]) * v[1] for i in range(len(W))]

    silu = lambda t: t / (1 + math.exp(-t))
    xs = [[3.0, 4.0], [1.0, 0.0]]
    vs = [mv(Wv, norm(x)) for x in xs]
    want = []
    for r, x in enumerate(xs):
        vis = vs[:r + 1]
        o = [sum(v[0] for v in vis) / len(vis), sum(v[1] for v in vis) / len(vis)]
        x = [x[0] + mv(Wo, o)[0], x[1] + mv(Wo, o)[1]]
        h = norm(x, (2.0, 1.0))
        g, u = mv(Wg, h), mv(Wu, h)
        a = [silu(g[0]) * u[0], silu(g[1]) * u[1]]
        dn = mv(Wd, a)
        x = [x[0] + dn[0], x[1] + dn[1]]
        want.append(mv(LM, norm(x)))
    np.testing.assert_allclose(z, np.array(want), rtol=2e-6, atol=2e-6)
    # keys are stored rotated: position 0 unrotated, position 1 rotated by angle 1 (theta_0 = 1)
    k1 = norm(xs[1])
    np.testing.assert_allclose(s.K[0][1, 0], [k1[0] * math.cos(1) - k1[1] * math.sin(1),
                                             k1[1] * math.cos(1) + k1[0] * math.sin(1)], rtol=1e-6)
    np.testing.assert_allclose(s.K[0][0, 0], norm(xs[0]), rtol=1e-6)


def test_small_identities():
    g = np.array([0.5, -2.0, 3.0, 1.0], dtype=F32)
    np.testing.assert_allclose(rmsnorm(np.full((1, 4), 7.0, F32), g, 0.0)[0], g, rtol=1e-6)
    np.testing.assert_allclose(rmsnorm(np.full((1, 4), -7.0, F32), g, 0.0)[0], -g, rtol=1e-6)
    rng = np.random.default_rng(0)
    z = rng.standard_normal((3, 50)).astype(F32)
    np.testing.assert_allclose(softmax_rows(z), softmax_rows(z + F32(13.5)), atol=1e-6)
    np.testing.assert_allclose(softmax_rows(z).sum(axis=1), 1.0, atol=1e-6)
    v = rng.standard_normal((5, 3, 16)).astype(F32)
    c0, s0 = rope_tables(np.zeros(5, dtype=np.int64), 16, 10000.0)
    np.testing.assert_array_equal(rope(v, c0, s0), v)
    c, s = rope_tables(np.arange(5) + 100, 16, 10000.0)
    np.testing.assert_allclose(np.linalg.norm(rope(v, c, s), axis=-1), np.linalg.norm(v, axis=-1), rtol=1e-5)
    # scores depend on the position difference only
    q, k = v[:1, :1], v[1:2, :1]
    def score(pq, pk):
        cq, sq = rope_tables(np.array([pq]), 16, 10000.0)
        ck, sk = rope_tables(np.array([pk]), 16, 10000.0)
        return float((rope(q, cq, sq) * rope(k, ck, sk)).sum())
    assert abs(score(17, 5) - score(112, 100)) < 1e-4
    assert abs(score(17, 5) - score(5, 17)) > 1e-3
    # first frequency is 1 rad per position, last pair rotates slowest
    c1, s1 = rope_tables(np.array([1]), 16, 10000.0)
    assert abs(c1[0, 0] - math.cos(1.0)) < 1e-7 and abs(s1[0, 7] - math.sin(10000.0 ** (-14 / 16))) < 1e-7


def _seq_with_prefix(m, n=20, max_len=64, seed=6):
    s = OracleSeq(m, max_len)
    s.prefill(I.make_tokens(n, m.s.vocab, seed), chunk=7)
    return s


def test_verify_commits_accepted_plus_one_and_rollback_reproduces():
    m = _model()
    s = _seq_with_prefix(m)
    k = 5
    d, q = I.make_independent_drafts(k, SMALL.vocab, 10, 11, scale=0.5)
    u = I.make_uniforms(k + 1, 12)
    lp = s.prefix_len
    a, nxt = s.nav_verify(d, q, u)
    assert s.prefix_len == lp + a + 1 and s.cached == lp + a and s.committed[-1] == nxt
    assert s.committed[lp:lp + a] == [int(t) for t in d[:a]]
    s.rollback(lp)
    assert s.prefix_len == lp and s.cached == lp - 1
    assert s.nav_verify(d, q, u) == (a, nxt)


def test_state_after_rounds_equals_fresh_prefill_of_committed_text():
    m = _model()
    s = _seq_with_prefix(m)
    for r in range(4):
        d, q = I.make_independent_drafts(4, SMALL.vocab, 20 + r, 30 + r, scale=0.3)
        s.nav_verify(d, q, I.make_uniforms(5, 40 + r))
    probe = I.make_tokens(3, SMALL.vocab, 50)
    z1 = s.forward_logits(probe)
    f = OracleSeq(m, 64)
    f.prefill(s.committed, chunk=64)
    z2 = f.forward_logits(probe)
    assert np.abs(z1 - z2).max() < 1e-5 * max(1.0, np.abs(z1).max())


def test_greedy_verify_matches_sequential_argmax_decoding():
    """Token matching: the committed text equals what plain one-token-at-a-time argmax decoding
    of the target would have produced (Sec. 2.2)."""
    m = _model()
    base = I.make_tokens(10, SMALL.vocab, 8)
    ar = OracleSeq(m, 64)
    ar.prefill(base, chunk=64)
    text = list(ar.committed)
    for _ in range(8):
        z = ar.forward_logits([])
        t = int(np.argmax(z[0]))
        ar.cached += 1
        ar.committed.append(t)
    ref = ar.committed
    s = OracleSeq(m, 64)
    s.prefill(base, chunk=64)
    rng = np.random.default_rng(1)
    while s.prefix_len < len(ref):
        lp = s.prefix_len
        k = min(3, len(ref) - lp)
        d = np.array(ref[lp:lp + k])
        if rng.random() < 0.5:
            j = rng.integers(0, k)
            d[j] = (d[j] + 1) % SMALL.vocab
        s.nav_verify(d, None, None)
    assert s.committed[:len(ref)] == ref


def _greedy_text(m, base, n):
    """n tokens of plain one-token-at-a-time argmax decoding after `base`."""
    ar = OracleSeq(m, 96)
    ar.prefill(base, chunk=64)
    for _ in range(n):
        t = int(np.argmax(ar.forward_logits([])[0]))
        ar.cached += 1
        ar.committed.append(t)
    return ar.committed


def test_chained_rounds_on_proactive_buffers_equal_plain_greedy_decoding():
    """Appendix B: buffers whose first token is the extra token the target produces, and whose
    other tokens are what the target would generate, stay valid round after round; the committed
    text is then plain argmax decoding, one round's k + 1 tokens at a time."""
    m = _model()
    base = I.make_tokens(9, SMALL.vocab, 21)
    ref = _greedy_text(m, base, 14)
    n0 = len(base)
    # round 0: 3 drafts (+ extra token = ref[n0 + 3]); buffer 1: guess ref[n0 + 3] + 4 drafts; buffer 2: guess + 2 drafts
    rounds = [(ref[n0:n0 + 3], None, None), (ref[n0 + 3:n0 + 8], None, None), (ref[n0 + 8:n0 + 11], None, None)]
    s = OracleSeq(m, 96)
    s.prefill(base, chunk=64)
    out = s.nav_verify_chain(rounds)
    assert [a for a, _ in out] == [3, 4, 2]
    assert s.committed == ref[:n0 + 3 + 1 + 4 + 1 + 2 + 1]
    assert [nx for _, nx in out] == [ref[n0 + 3], ref[n0 + 8], ref[n0 + 11]]


def test_chain_stops_at_a_wrong_guess_or_a_rejected_draft_and_leaves_the_state_of_the_last_round():
    m = _model()
    base = I.make_tokens(9, SMALL.vocab, 21)
    ref = _greedy_text(m, base, 14)
    n0 = len(base)
    wrong = (ref[n0 + 3] + 1) % SMALL.vocab
    # (i) wrong guess of the extra token: only round 0 runs
    s = OracleSeq(m, 96)
    s.prefill(base, chunk=64)
    out = s.nav_verify_chain([(ref[n0:n0 + 3], None, None), ([wrong] + ref[n0 + 4:n0 + 8], None, None)])
    assert out == [(3, ref[n0 + 3])] and s.committed == ref[:n0 + 4] and s.cached == n0 + 3
    # (ii) a rejected draft in round 0: its buffer is dropped even though the guess equals the correction
    bad = list(ref[n0:n0 + 3])
    bad[1] = (bad[1] + 1) % SMALL.vocab
    s = OracleSeq(m, 96)
    s.prefill(base, chunk=64)
    out = s.nav_verify_chain([(bad, None, None), ([ref[n0 + 1]] + ref[n0 + 2:n0 + 5], None, None)])
    assert out == [(1, ref[n0 + 1])] and s.committed == ref[:n0 + 2]
    # (iii) the same rounds given one by one, with the validity rule applied by hand, end in the same state
    t = OracleSeq(m, 96)
    t.prefill(base, chunk=64)
    assert t.nav_verify(bad, None, None) == (1, ref[n0 + 1]) and t.committed == s.committed and t.cached == s.cached


def test_chain_with_the_sampling_rule_keeps_buffers_exactly_when_the_rule_says():
    """q == p makes every draft accepted whatever the uniforms are (ratio 1), so the chain goes on
    exactly when the buffer's first token is the extra token drawn from p_{k+1}."""
    m = _model()
    base = I.make_tokens(7, SMALL.vocab, 33)
    probe = OracleSeq(m, 96)
    probe.prefill(base, chunk=64)
    d0 = I.make_tokens(3, SMALL.vocab, 34)
    p0 = softmax_rows(probe.forward_logits(d0))
    u0 = I.make_uniforms(4, 35)
    a0, x0 = probe.nav_verify(d0, p0[:3].copy(), u0)
    assert a0 == 3
    d1 = I.make_tokens(2, SMALL.vocab, 36)
    p1 = softmax_rows(probe.forward_logits(d1))
    u1 = I.make_uniforms(3, 37)
    a1, x1 = probe.nav_verify(d1, p1[:2].copy(), u1)
    s = OracleSeq(m, 96)
    s.prefill(base, chunk=64)
    out = s.nav_verify_chain([(d0, p0[:3].copy(), u0), ([x0] + list(d1), p1[:2].copy(), u1)])
    assert out == [(a0, x0), (a1, x1)] and s.committed == probe.committed
    s = OracleSeq(m, 96)
    s.prefill(base, chunk=64)
    out = s.nav_verify_chain([(d0, p0[:3].copy(), u0), ([(x0 + 1) % SMALL.vocab] + list(d1), p1[:2].copy(), u1)])
    assert out == [(a0, x0)] and s.prefix_len == len(base) + 4
