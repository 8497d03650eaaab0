#!/usr/bin/env python3
"""Writes tests/golden/llama8b_nav.json: what the CPU checker computes for the full 32-layer 8B-shape
workload (2048-token prefix, k = 8).  Calls only oracle/ and the seeded input generators; takes
tens of minutes and ~40 GB of host memory.  Run from the repository root:
    python tests/golden/make_llama8b_golden.py
"""
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle.nav import OracleSeq  # noqa: E402
from oracle.spec_sampling import accept_test  # noqa: E402
from oracle.transformer import OracleModel, softmax_rows  # noqa: E402
from paper_2605_13319_amd import inputs as I  # noqa: E402

N_SAMPLES = 48


def main():
    wl = I.WORKLOADS["llama-8b"]
    shape, seed, prefix, k = wl["shape"], wl["seed"], wl["prefix"], wl["k"]
    t0 = time.time()
    w = I.make_weights(shape, seed + I.SEED_WEIGHTS)
    print(f"weights {time.time() - t0:.0f}s", flush=True)
    toks = I.make_tokens(prefix, shape.vocab, seed + I.SEED_PREFIX)
    seq = OracleSeq(OracleModel(shape, w), prefix + 64)
    seq.prefill(toks, chunk=4096)
    print(f"prefill {time.time() - t0:.0f}s", flush=True)

    # pass A, token matching: the checker's own argmax continuation, broken at draft 6
    d = []
    for i in range(k):
        d.append(int(np.argmax(seq.forward_logits(d)[-1])))
        print(f"draft {i} {time.time() - t0:.0f}s", flush=True)
    d[5] = (d[5] + 12345) % shape.vocab
    z = seq.forward_logits(d)
    rng = np.random.default_rng(seed + 99)
    samples = []
    for r in range(k + 1):
        idx = sorted(set(int(i) for i in rng.integers(0, shape.vocab, N_SAMPLES)) | {int(np.argmax(z[r]))})
        samples.append({"row": r, "idx": idx, "val": [float(z[r, i]) for i in idx]})
    top2 = np.sort(z, axis=1)[:, -2:]
    lp = seq.prefix_len
    a_greedy, n_greedy = seq.nav_verify(np.array(d, dtype=np.int32), None, None)
    seq.rollback(lp)

    # pass B, stochastic rule with draft distributions that ignore the target
    d2, q2 = I.make_independent_drafts(k, shape.vocab, seed + I.SEED_NOISE, seed + I.SEED_DRAFT_U, scale=1.0)
    u2 = I.make_uniforms(k + 1, seed + I.SEED_VERIFY_U)
    p2 = softmax_rows(seq.forward_logits(d2))
    ratios = [float(p2[i, d2[i]]) / float(q2[i, d2[i]]) for i in range(k)]
    a_spec, n_spec = seq.nav_verify(d2, q2, u2)
    seq.rollback(lp)
    # the one draw of pass B: every token whose interval of the draw's CDF (residual of row a, or the
    # extra-token row) comes within 1e-3 of the uniform is a result the end-to-end rule excuses
    w_row = np.maximum(np.float32(0.0), p2[a_spec] - q2[a_spec]) if a_spec < k else p2[k]
    cdf = np.cumsum(w_row.astype(np.float64))
    cdf /= cdf[-1]
    lo = np.concatenate([[0.0], cdf[:-1]])
    u_draw = float(u2[k])
    near = np.nonzero((cdf > u_draw - 1e-3) & (lo < u_draw + 1e-3) & (w_row > 0))[0]
    assert n_spec in near

    out = {
        "workload": "llama-8b", "prefix": prefix, "k": k, "seed": seed,
        "pass_a": {"drafts": d, "accepted_len": a_greedy, "next_token": n_greedy, "samples": samples,
                   "row_argmax": [int(i) for i in np.argmax(z, axis=1)],
                   "row_top2_gap": [float(t[1] - t[0]) for t in top2]},
        "pass_b": {"draft_scale": 1.0, "accepted_len": a_spec, "next_token": n_spec,
                   "ratios": ratios, "uniforms": [float(x) for x in u2],
                   "next_token_within_1e-3_of_the_uniform": [int(i) for i in near]},
    }
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "llama8b_nav.json")
    with open(path, "w") as f:
        json.dump(out, f, indent=1)
    print(f"wrote {path} after {time.time() - t0:.0f}s", flush=True)


if __name__ == "__main__":
    main()
