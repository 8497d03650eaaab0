"""Batched verification of several clients in one call (the multi-client case of Appendix I, with
lengths and k drawn per client and per round as the dual-threshold trigger would produce them):
per client the result and the state afterwards must be those of a single-client pass."""
import numpy as np
import pytest

from oracle.transformer import softmax_rows
from paper_2605_13319_amd import inputs as I
from tests.helpers import decision_excused, drafts_from_oracle, oracle_side

pytestmark = pytest.mark.gpu

SMALL_BF16 = I.ModelShape("small-bf16", 3, 512, 8, 2, 64, 1024, 2048)


@pytest.fixture(scope="module")
def nav():
    import torch
    assert torch.cuda.is_available()
    from paper_2605_13319_amd import nav as n
    return n


# vocabulary 24581 = 1537 n-tiles: the last tile is ragged (5 of 16 rows), the last group of 8 tiles
# holds one tile, and the LM head of a pass of more than 64 rows runs whole-K workgroups
RAGGED_BF16 = I.ModelShape("ragged-bf16", 2, 512, 8, 2, 64, 1024, 24581)


# the 8B widths with two layers: the shapes the 16-client workload runs (K = 4096 in 8 slices, the
# down projection's K = 14336 in 7 x 4, 128256 vocabulary columns) at its prefix lengths
LLAMA_8B_L2 = I.WORKLOADS["llama-8b"]["shape"].truncated(2)


@pytest.mark.parametrize("shape_name,n_seq,rounds,max_prefix", [("tiny", 5, 4, 150), ("small-bf16", 5, 4, 150),
                                                                 ("small-bf16", 16, 12, 150), ("ragged-bf16", 16, 3, 150),
                                                                 ("llama-8b-L2", 16, 10, 4096),
                                                                 ("llama-13b-L2", 16, 3, 600)])
def test_batched_call_equals_single_calls_bit_for_bit(nav, shape_name, n_seq, rounds, max_prefix):
    """bf16: the clients' rows share passes of up to 256 rows (16 clients with k ~ U[1,16] bring about
    150: beyond 128 rows the packed activations have 16 row tiles and the wide GEMM its second shape;
    at the 13B widths, K = 5120 = 5 x 2 slices, the whole-K products fall back to the narrow kernel
    on up to 16 row tiles); a row's results must not depend on what else is in its pass."""
    shape = {"tiny": I.WORKLOADS["tiny"]["shape"], "small-bf16": SMALL_BF16, "ragged-bf16": RAGGED_BF16,
             "llama-8b-L2": LLAMA_8B_L2, "llama-13b-L2": I.WORKLOADS["llama-13b"]["shape"].truncated(2)}[shape_name]
    w = I.make_weights(shape, 9001)
    model = nav.Model(shape, w)
    rng = np.random.default_rng(9002)
    lens = [int(x) for x in rng.integers(17, max_prefix, n_seq)]
    per_seq = (max_prefix + 17 * rounds) // 16 + 4
    kv_b = nav.KVCache(model, max_seqs=n_seq, n_blocks=per_seq * n_seq)
    kv_s = nav.KVCache(model, max_seqs=n_seq, n_blocks=per_seq * n_seq)
    for s, n in enumerate(lens):
        toks = I.make_tokens(n, shape.vocab, 9100 + s)
        kv_b.prefill(s, toks)
        kv_s.prefill(s, toks)
    for rnd in range(rounds):
        ks = [int(x) for x in rng.integers(1, 17, n_seq)]
        fixed = {0: 15, 1: 11, 2: 13, 3: 9, 4: 16}
        if n_seq == 16 and rnd in fixed and rnd < rounds - 1:
            # passes of 256, 192, 224 and 160 rows: each staged-row-tile shape of the wide GEMM, all tiles
            # live; 272 rows: more than a pass holds (15 clients in one pass, the last in a second)
            ks = [fixed[rnd]] * n_seq
        drafts, probs, us = [], [], []
        for s in range(n_seq):
            d, q = I.make_independent_drafts(ks[s], shape.vocab, 9200 + 100 * rnd + s, 9300 + 100 * rnd + s, scale=1.0)
            drafts.append([int(t) for t in d])
            greedy = (s == 2)  # one client uses token matching
            probs.append(None if greedy else q)
            us.append(None if greedy else I.make_uniforms(ks[s] + 1, 9400 + 100 * rnd + s))
        order = [int(x) for x in rng.permutation(n_seq)]  # clients in any order
        a_b, n_b = kv_b.nav_verify_batch(order, [drafts[s] for s in order], [probs[s] for s in order],
                                         [us[s] for s in order])
        for i, s in enumerate(order):
            a, n = kv_s.nav_verify(s, drafts[s], probs[s], us[s])
            assert (a_b[i], n_b[i]) == (a, n), (rnd, s)
            assert kv_b.length(s) == kv_s.length(s) == lens[s] + a + 1
            assert kv_b.seq_blocks(s) == kv_s.seq_blocks(s)
            lens[s] += a + 1
        assert kv_b.free_blocks() == kv_s.free_blocks()
    # the caches hold the same values
    for s in range(n_seq):
        for layer in range(shape.n_layers):
            for pos in (0, lens[s] // 2, lens[s] - 2):
                kb, vb = kv_b.read_kv(s, layer, pos)
                ks_, vs = kv_s.read_kv(s, layer, pos)
                np.testing.assert_array_equal(kb, ks_)
                np.testing.assert_array_equal(vb, vs)


def test_batched_call_that_cannot_get_its_blocks_changes_nothing(nav):
    shape = SMALL_BF16
    model = nav.Model(shape, I.make_weights(shape, 9001))
    kv = nav.KVCache(model, max_seqs=3, n_blocks=7)
    for s, n in enumerate((31, 32, 30)):  # 2 blocks each: 6 of 7 in use; each client needs one more for 16 drafts
        kv.prefill(s, I.make_tokens(n, shape.vocab, 9500 + s))
    free0 = kv.free_blocks()
    assert free0 == 1
    d = [[1] * 16, [2] * 16, [3] * 16]
    with pytest.raises(nav.PipesdError) as e:
        kv.nav_verify_batch([0, 1, 2], d)
    assert e.value.status == nav.ENOMEM
    assert kv.free_blocks() == free0 and [kv.length(s) for s in range(3)] == [31, 32, 30]
    a, n = kv.nav_verify_batch([1], [d[1]])  # one client alone still fits
    assert kv.length(1) == 32 + a[0] + 1


def test_batched_rounds_against_the_checker(nav):
    """Four clients with their own prefixes, three rounds of k ~ U[1,16] noisy-target drafts: every
    decision is the checker's (or excused by the end-to-end rule) and the lengths follow."""
    shape = SMALL_BF16
    w = I.make_weights(shape, 9601)
    model = nav.Model(shape, w)
    n_seq = 4
    rng = np.random.default_rng(9602)
    lens = [int(x) for x in rng.integers(20, 120, n_seq)]
    kv = nav.KVCache(model, max_seqs=n_seq, n_blocks=64)
    oseqs = []
    for s, n in enumerate(lens):
        toks = I.make_tokens(n, shape.vocab, 9610 + s)
        kv.prefill(s, toks)
        oseqs.append(oracle_side(shape, w, toks, n + 80))
    for rnd in range(3):
        ks = [int(x) for x in rng.integers(1, 17, n_seq)]
        drafts, probs, us, refs, prows = [], [], [], [], []
        for s in range(n_seq):
            d, q = drafts_from_oracle(oseqs[s], ks[s], 0.5, 9700 + 10 * rnd + s, 9800 + 10 * rnd + s)
            u = I.make_uniforms(ks[s] + 1, 9900 + 10 * rnd + s)
            drafts.append([int(t) for t in d]); probs.append(q); us.append(u)
            prows.append(softmax_rows(oseqs[s].forward_logits(d)))
            refs.append(oseqs[s].nav_verify(d, q, u))
        a_b, n_b = kv.nav_verify_batch(list(range(n_seq)), drafts, probs, us)
        for s in range(n_seq):
            a_ref, n_ref = refs[s]
            if (a_b[s], n_b[s]) != (a_ref, n_ref):
                assert a_b[s] != a_ref and decision_excused(prows[s], probs[s], drafts[s], us[s], a_b[s], a_ref), \
                    f"round {rnd} client {s}: {(a_b[s], n_b[s])} vs checker {(a_ref, n_ref)}"
                o = oseqs[s]
                o.rollback(lens[s])
                o.committed += drafts[s][:a_b[s]] + [n_b[s]]
                o.cached = lens[s] + a_b[s]
            lens[s] += a_b[s] + 1
            assert kv.length(s) == lens[s] == oseqs[s].prefix_len


def test_fifty_growing_rounds_of_sixteen_clients_against_the_checker(nav):
    """The multi-client workload as it is written (Appendix I; 16 clients, per-client prefixes, k ~
    U[1,16] redrawn every round as the dual-threshold trigger would, drafts q = softmax(target logits
    + 0.5 N) from the checker's own logits, 50 consecutive verify / rollback rounds) at a small shape:
    the sequences GROW by accepted + 1 tokens per round, every decision of every round equals the
    checker's or is excused by the 1e-3 rule, and lengths and block counts follow."""
    shape = SMALL_BF16
    w = I.make_weights(shape, 9651)
    model = nav.Model(shape, w)
    n_seq, rounds = 16, 50
    rng = np.random.default_rng(9652)
    lens = [int(x) for x in rng.integers(17, 150, n_seq)]
    max_len = 150 + 17 * rounds + 32
    kv = nav.KVCache(model, max_seqs=n_seq, n_blocks=n_seq * (max_len // 16 + 2))
    oseqs = []
    for s, n in enumerate(lens):
        toks = I.make_tokens(n, shape.vocab, 9660 + s)
        kv.prefill(s, toks)
        oseqs.append(oracle_side(shape, w, toks, max_len))
    excused = accepted = drafted = 0
    for rnd in range(rounds):
        ks = [int(x) for x in rng.integers(1, 17, n_seq)]
        drafts, probs, us, refs, prows = [], [], [], [], []
        for s in range(n_seq):
            d, q = drafts_from_oracle(oseqs[s], ks[s], 0.5, 20000 + 100 * rnd + s, 30000 + 100 * rnd + s)
            u = I.make_uniforms(ks[s] + 1, 40000 + 100 * rnd + s)
            drafts.append([int(t) for t in d]); probs.append(q); us.append(u)
            prows.append(softmax_rows(oseqs[s].forward_logits(d)))
            refs.append(oseqs[s].nav_verify(d, q, u))
        a_b, n_b = kv.nav_verify_batch(list(range(n_seq)), drafts, probs, us)
        for s in range(n_seq):
            a_ref, n_ref = refs[s]
            if (a_b[s], n_b[s]) != (a_ref, n_ref):
                assert a_b[s] != a_ref and decision_excused(prows[s], probs[s], drafts[s], us[s], a_b[s], a_ref), \
                    f"round {rnd} client {s}: {(a_b[s], n_b[s])} vs checker {(a_ref, n_ref)}"
                excused += 1
                o = oseqs[s]
                o.rollback(lens[s])
                o.committed += drafts[s][:a_b[s]] + [n_b[s]]
                o.cached = lens[s] + a_b[s]
            lens[s] += a_b[s] + 1
            accepted += a_b[s]
            drafted += ks[s]
            assert kv.length(s) == lens[s] == oseqs[s].prefix_len
            assert kv.seq_blocks(s) == (lens[s] - 1 + 15) // 16
        if rnd % 10 == 9:
            print(f"round {rnd}: lengths {min(lens)}..{max(lens)}, accepted {accepted}/{drafted}, excused {excused}", flush=True)
    assert sum(lens) > sum(int(x) for x in np.random.default_rng(9652).integers(17, 150, n_seq)) + n_seq * rounds
    assert excused <= 3, excused
