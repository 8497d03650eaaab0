#!/usr/bin/env python3
"""Benchmark of the NAV pass on one MI355X.

A step = one whole pass of the hot path for one client: forward of [pending, d_1..d_k] over the
paged KV cache, softmax, accept tests, corrected/extra-token draw, KV trim, then the host-side
rollback to the starting prefix so every step does identical work.  Inputs (weights, prefilled
cache, draft distributions) are resident in HBM before the timed region.

Prints ONE JSON line: verified tokens/s (k / t_pass), ms per pass (mean; median and p10/p90 beside
it), the algorithmic HBM rate of the whole pass, a `roofline` object for the weight-streaming GEMM
kernel measured with HIP events in the timed region (its `traffic` comes from the committed
counter summary under profiles/ and is null once the kernel sources have changed since), and a
`cpu_baseline` object: the CPU checker timed on this host on a layer-truncated sample of the same
workload.
"""
import argparse
import hashlib
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 matrix-core peak of the device


def log(*a):
    print(*a, file=sys.stderr, flush=True)


GEMM_SOURCES = ("device_gemm.h", "kernels_gemm.hip", "common.h")
TRAFFIC_SUMMARY = os.path.join(ROOT, "profiles", "nav_pass_llama8b_k8_per_projection.md")


def gemm_sources_sha():
    h = hashlib.sha256()
    for fn in GEMM_SOURCES:
        with open(os.path.join(ROOT, "paper_2605_13319_amd", "csrc", fn), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def committed_traffic(workload, projection):
    """HBM bytes per launch of the given projection's kernel from the committed counter summary, or
    None if there is none for this workload or the GEMM sources have changed since the counters
    were taken."""
    if workload != "llama-8b" or not os.path.exists(TRAFFIC_SUMMARY):
        return None
    txt = open(TRAFFIC_SUMMARY).read()
    sha = re.search(r"sources-sha256:\s*([0-9a-f]{64})", txt)
    val = re.search(r"traffic-bytes-per-launch\[" + re.escape(projection) + r"\]:\s*([0-9.eE+]+)", txt)
    if not sha or not val or sha.group(1) != gemm_sources_sha():
        return None
    return float(val.group(1))


def cpu_baseline(shape, weights, prefix, k, layers):
    """The checker's verify pass (k + 1 rows over an already-cached prefix + decision) on a model
    truncated to `layers` layers; layer time is scaled to the full depth, head time added once."""
    import numpy as np
    from oracle.nav import OracleSeq
    from oracle.spec_sampling import spec_accept
    from oracle.transformer import OracleModel, softmax_rows
    from paper_2605_13319_amd import inputs as I
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    small = shape.truncated(layers)
    w = dict(weights)
    for name in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "attn_norm", "ffn_norm"):
        w[name] = weights[name][:layers]
    om = OracleModel(small, w)
    seq = OracleSeq(om, prefix + k + 1)
    rng = np.random.default_rng(1)
    for l in range(layers):  # timing does not depend on the cached values
        seq.K[l][:prefix - 1] = rng.standard_normal(seq.K[l][:prefix - 1].shape, dtype=np.float32)
        seq.V[l][:prefix - 1] = rng.standard_normal(seq.V[l][:prefix - 1].shape, dtype=np.float32)
    seq.committed = [0] * prefix
    seq.cached = prefix - 1
    d, q = I.make_independent_drafts(k, shape.vocab, 11, 12, scale=1.0)
    u = I.make_uniforms(k + 1, 13)
    # layers-only time: same model without the head is not expressible in the checker, so time the
    # full truncated pass and a 0-layer pass (embedding + head + decision) and subtract
    head = OracleModel(shape.truncated(0), w)
    hseq = OracleSeq(head, 4)
    hseq.committed = [0]

    def timed(fn, reps):
        ts = []
        for _ in range(reps):
            t0 = time.perf_counter()
            fn()
            ts.append(time.perf_counter() - t0)
        return sorted(ts)[len(ts) // 2]

    def full():
        z = seq.forward_logits(d)
        spec_accept(softmax_rows(z), q, d, u)

    def head_only():
        z = hseq.forward_logits(d)
        spec_accept(softmax_rows(z), q, d, u)

    t_full = timed(full, 3)
    t_head = timed(head_only, 3)
    t_layer = max(t_full - t_head, 0.0) / layers
    t_pass = t_layer * shape.n_layers + t_head
    return {"value": k / t_pass, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "ms_per_pass": t_pass * 1e3,
            "sample": f"{layers}-layer truncation of {shape.name} (full width, vocab, ctx {prefix}, k={k}); "
                      f"per-layer time x {shape.n_layers} + head/decision time; median of 3"}


def run_batched(np, torch, I, nav, model, shape, seed, lens, rounds, warmup, sigma, k_of, grow=True):
    """Several clients per call (the multi-client setting of Appendix I) on a model that is already
    on the device: client s starts from a prefix of lens[s] tokens; every round it brings k_of(round,
    s) drafts with q_i = softmax(target logits + sigma N(0,1)), d_i ~ q_i (the target logits are the
    library's own: draft generation is outside the timed region), all clients are verified by ONE
    pipesd_nav_verify_batch call, and (grow) the sequences keep what the call committed, so they grow
    by accepted + 1 tokens per round.  Returns the timing record of the `rounds` timed calls."""
    n_seq = len(lens)
    lens = list(lens)
    kv = nav.KVCache(model, n_seq, sum((n + 17 * (rounds + warmup) + 64) // 16 + 2 for n in lens))
    t0 = time.time()
    for s, n in enumerate(lens):
        kv.prefill(s, I.make_tokens(n, shape.vocab, seed + 100 + s))
    torch.cuda.synchronize()
    log(f"[bench] {n_seq} prefixes ({sum(lens)} tokens) cached in {time.time() - t0:.1f}s")
    esz = 4 if shape.dtype == I.DTYPE_F32 else 2
    w_bytes = shape.n_params_streamed() * esz
    times, ks_sum, rows, alg, committed = [], 0, [], 0.0, 0
    start_lens = list(lens)
    for r in range(warmup + rounds):
        ks = [k_of(r, s) for s in range(n_seq)]
        drafts, probs, us = [], [], []
        for s in range(n_seq):
            if sigma is None:
                d, q = I.make_independent_drafts(ks[s], shape.vocab, seed + 1000 * r + s, seed + 1000 * r + 500 + s, scale=1.0)
            else:
                d, q = I.make_noisy_target_drafts(lambda ds, s=s: kv.forward_logits(s, ds)[-1], ks[s], shape.vocab, sigma,
                                                  seed + 1000 * r + s, seed + 1000 * r + 500 + s)
            drafts.append([int(t) for t in d])
            probs.append(torch.from_numpy(q).cuda())
            us.append(I.make_uniforms(ks[s] + 1, seed + 7 + 100 * r + s))
        torch.cuda.synchronize()
        t = time.perf_counter()
        a, _ = kv.nav_verify_batch(list(range(n_seq)), drafts, probs, us)
        dt = time.perf_counter() - t
        if r >= warmup:
            times.append(dt)
            ks_sum += sum(ks)
            committed += sum(a) + n_seq  # every client commits its accepted drafts and one more token
            rows.append(sum(ks) + n_seq)
            # weights once per call; per client the cached K/V read, the new rows written and q read
            alg += w_bytes + sum(shape.algorithmic_bytes(lens[s], ks[s]) - w_bytes for s in range(n_seq))
        for s in range(n_seq):
            if grow:
                lens[s] += a[s] + 1
            else:
                kv.rollback(s, lens[s])
    total = sum(times)
    kv.close()
    return {"ms_per_call": total / len(times) * 1e3, "verified_tokens_per_sec": ks_sum / total,
            "committed_tokens_per_sec": committed / total, "hbm_algorithmic_gbps": alg / total / 1e9,
            "hbm_frac_of_peak": alg / total / 1e9 / HBM_PEAK_GBPS, "mean_rows_per_call": float(np.mean(rows)),
            "acceptance_rate": (committed - n_seq * len(times)) / max(ks_sum, 1), "calls": len(times),
            "prefix_tokens_at_start": sum(start_lens), "prefix_tokens_at_end": sum(lens),
            "ms_per_call_median_p10_p90": [float(np.percentile(times, q)) * 1e3 for q in (50, 10, 90)]}


def batched(args, np, torch, I, nav):
    """--batch N: the multi-client call on its own (prefixes U[256,4096] unless --prefix, k U[1,16]
    redrawn every round unless --k or --trigger, noisy-target drafts, sequences that grow)."""
    wl = I.WORKLOADS[args.workload]
    shape = wl["shape"] if args.layers is None else wl["shape"].truncated(args.layers)
    seed = wl["seed"] + 1000
    n_seq = args.batch
    weights = I.make_weights(shape, wl["seed"] + I.SEED_WEIGHTS, threads=min(16, os.cpu_count() or 8))
    model = nav.Model(shape, weights)
    rng = np.random.default_rng(seed + I.SEED_LENGTHS)
    lens = [args.prefix] * n_seq if args.prefix else [int(x) for x in rng.integers(256, 4097, n_seq)]
    n_rounds = args.warmup + args.steps
    if args.trigger:
        r1, r2 = (float(x) for x in args.trigger.split(","))
        traces = []
        for s in range(n_seq):  # 16 = the longest draft a client sends in this workload
            lens_s, _ = nav.trigger_rounds(I.make_confidences(16 * n_rounds, seed + 300 + s), r1, r2, 16, cap=n_rounds)
            assert len(lens_s) == n_rounds
            traces.append(lens_s)
        k_of = lambda r, s: traces[s][r]
    elif args.k:
        k_of = lambda r, s: args.k
    else:
        ks_all = rng.integers(1, 17, (n_rounds, n_seq))
        k_of = lambda r, s: int(ks_all[r, s])
    sigma = None if args.independent_drafts else wl["sigma"]
    rec = run_batched(np, torch, I, nav, model, shape, seed, lens, args.steps, args.warmup, sigma, k_of,
                      grow=not args.no_grow)
    esz = 4 if shape.dtype == I.DTYPE_F32 else 2
    out = {
        "metric": "verified_tokens_per_sec", "value": rec["verified_tokens_per_sec"], "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": rec["ms_per_call"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if esz == 2 else "f32", "data": "synthetic",
        "config": {"workload": f"{shape.name}: {n_seq} clients per call, prefixes "
                               + (f"{args.prefix}" if args.prefix else "U[256,4096]") + ", k "
                               + (f"from the dual-threshold trigger (R1,R2 = {args.trigger}) on Beta(8,1) confidences"
                                  if args.trigger else f"{args.k}" if args.k else "U[1,16] redrawn every round")
                               + (", drafts independent of the target" if sigma is None else f", drafts softmax(target + {sigma} N)")
                               + (", every round from the same prefixes" if args.no_grow else ", sequences grow over the rounds")
                               + ", paged KV (16-token blocks)", "mean_rows_per_call": rec["mean_rows_per_call"]},
        "committed_tokens_per_sec": rec["committed_tokens_per_sec"],
        "hbm_algorithmic_gbps": rec["hbm_algorithmic_gbps"], "hbm_frac_of_peak": rec["hbm_frac_of_peak"],
        "acceptance_rate": rec["acceptance_rate"],
        "ms_per_step_median_p10_p90": rec["ms_per_call_median_p10_p90"],
        "roofline": None,
    }
    print(json.dumps(out), flush=True)


def single_client_record(np, torch, I, nav, model, shape, seed, prefix, k, sigma, steps, warmup, kv=None):
    """ms per pass, verified tokens/s and algorithmic HBM rate of the single-client pass on a model
    that is already on the device (drafts from the library's own logits, outside the timed region)."""
    own = kv is None
    if own:
        kv = nav.KVCache(model, max_seqs=1, n_blocks=(prefix + nav.MAX_ROWS + 15) // 16 + 2)
        kv.prefill(0, I.make_tokens(prefix, shape.vocab, seed + I.SEED_PREFIX))
    if sigma is None:
        d, q = I.make_independent_drafts(k, shape.vocab, seed + I.SEED_NOISE, seed + I.SEED_DRAFT_U)
    else:
        d, q = I.make_noisy_target_drafts(lambda ds: kv.forward_logits(0, ds)[-1], k, shape.vocab, sigma,
                                          seed + I.SEED_NOISE + k, seed + I.SEED_DRAFT_U + k)
    q_dev = torch.from_numpy(q).cuda()
    u = I.make_uniforms(k + 1, seed + I.SEED_VERIFY_U + k)
    times, acc = [], 0
    for r in range(warmup + steps):
        t = time.perf_counter()
        a, _ = kv.nav_verify(0, d, q_dev, u)
        dt = time.perf_counter() - t
        kv.rollback(0, prefix)
        if r >= warmup:
            times.append(dt)
            acc = a
    if own:
        kv.close()
    t_pass = sum(times) / len(times)
    alg = shape.algorithmic_bytes(prefix, k)
    return {"ms_per_pass": t_pass * 1e3, "verified_tokens_per_sec": k / t_pass, "committed_tokens_per_sec": (acc + 1) / t_pass,
            "hbm_algorithmic_gbps": alg / t_pass / 1e9, "hbm_frac_of_peak": alg / t_pass / 1e9 / HBM_PEAK_GBPS,
            "accepted_len": acc, "passes": len(times)}


def prefill(args, np, torch, I, nav):
    """Prompt ingestion (the step before the pass): n tokens into an empty sequence, which caches
    n - 1 rows and leaves the last one pending.  No LM head, no decision."""
    wl = I.WORKLOADS[args.workload]
    shape = wl["shape"] if args.layers is None else wl["shape"].truncated(args.layers)
    n = args.prefill
    weights = I.make_weights(shape, wl["seed"] + I.SEED_WEIGHTS, threads=min(16, os.cpu_count() or 8))
    model = nav.Model(shape, weights)
    kv = nav.KVCache(model, 1, (n + 15) // 16 + 2)
    toks = I.make_tokens(n, shape.vocab, wl["seed"] + I.SEED_PREFIX)
    times = []
    for r in range(args.warmup + args.steps):
        kv.reset(0)
        torch.cuda.synchronize()
        t = time.perf_counter()
        kv.prefill(0, toks)
        torch.cuda.synchronize()
        if r >= args.warmup:
            times.append(time.perf_counter() - t)
    total = sum(times)
    rows = n - 1
    # 2 flop per weight element and row (layer matrices only) + causal attention: row r scores r + 1
    # keys and weighs as many values, head_dim multiply-adds each, per query head and layer
    per_layer = (shape.q_dim + 2 * shape.kv_dim) * shape.d_model + shape.d_model * shape.q_dim + 3 * shape.d_ffn * shape.d_model
    flop = 2.0 * rows * shape.n_layers * per_layer + 4.0 * shape.n_layers * shape.q_dim * (rows * (rows + 1) / 2)
    achieved = flop * len(times) / total / 1e12
    out = {
        "metric": "prefill_tokens_per_sec", "value": rows * len(times) / total, "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": total / len(times) * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if shape.dtype != I.DTYPE_F32 else "f32", "data": "synthetic",
        "config": {"workload": f"{shape.name}: ingestion of a {n}-token prompt into an empty sequence, passes of up to "
                               f"128 rows, paged KV (16-token blocks)"},
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
                     "kernel": "all kernels of the call; algorithmic flop (each product counted once, not per bf16 half)"},
    }
    print(json.dumps(out), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="llama-8b")
    ap.add_argument("--k", type=int, default=None)
    ap.add_argument("--prefix", type=int, default=None)
    ap.add_argument("--layers", type=int, default=None, help="truncate the model (debugging; not the headline)")
    ap.add_argument("--cpu-layers", type=int, default=32)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy kernel (scale for the HBM byte counters)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--prof", default="all_gemm", help="kernel class bracketed by HIP events")
    ap.add_argument("--batch", type=int, default=0,
                    help="N > 0: time pipesd_nav_verify_batch on N clients instead (prefixes U[256,4096] unless --prefix, "
                         "k U[1,16] redrawn every round unless --k; --steps rounds).  An auxiliary line: no roofline / "
                         "cpu_baseline objects")
    ap.add_argument("--independent-drafts", action="store_true",
                    help="with --batch: drafts that ignore the target (acceptance near 0) instead of softmax(target + sigma N)")
    ap.add_argument("--no-grow", action="store_true",
                    help="with --batch: cut every client back to its prefix after each round instead of letting it grow")
    ap.add_argument("--no-extra", action="store_true",
                    help="leave out the `extra_configs` object (the other workloads of the configuration list)")
    ap.add_argument("--trigger", default=None,
                    help="with --batch: R1,R2 - every client's draft lengths come from the dual-threshold trigger "
                         "(Sec. 3.3) run over a seeded stream of synthetic confidences instead of U[1,16]")
    ap.add_argument("--prefill", type=int, default=0,
                    help="N > 0: time the ingestion of an N-token prompt instead (pipesd_prefill; --steps prompts).  "
                         "An auxiliary line: matrix-core roofline of the whole call, no cpu_baseline object")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: the NAV pass runs on ONE GPU; --gpus N with N > 1 is not supported")

    import numpy as np
    import torch
    from paper_2605_13319_amd import inputs as I
    from paper_2605_13319_amd import nav

    if args.batch > 0:
        return batched(args, np, torch, I, nav)
    if args.prefill > 0:
        return prefill(args, np, torch, I, nav)
    wl = I.WORKLOADS[args.workload]
    shape = wl["shape"] if args.layers is None else wl["shape"].truncated(args.layers)
    k = args.k or wl["k"]
    prefix = args.prefix or wl["prefix"]
    seed = wl["seed"]
    sigma = wl["sigma"]

    t0 = time.time()
    weights = I.make_weights(shape, seed + I.SEED_WEIGHTS, threads=min(16, os.cpu_count() or 8))
    log(f"[bench] weights for {shape.name} drawn in {time.time() - t0:.1f}s")
    t0 = time.time()
    model = nav.Model(shape, weights)
    n_blocks = (prefix + nav.MAX_ROWS + 15) // 16 + 2
    kv = nav.KVCache(model, max_seqs=1, n_blocks=n_blocks)
    toks = I.make_tokens(prefix, shape.vocab, seed + I.SEED_PREFIX)
    kv.prefill(0, toks)
    torch.cuda.synchronize()
    log(f"[bench] model on device and {prefix}-token prefix cached in {time.time() - t0:.1f}s")

    # drafts: q_i = softmax(target logits + sigma N(0,1)), d_i ~ q_i (fp32 model: independent drafts)
    if sigma is None:
        d, q = I.make_independent_drafts(k, shape.vocab, seed + I.SEED_NOISE, seed + I.SEED_DRAFT_U)
    else:
        d, q = I.make_noisy_target_drafts(lambda ds: kv.forward_logits(0, ds)[-1], k, shape.vocab, sigma,
                                          seed + I.SEED_NOISE, seed + I.SEED_DRAFT_U)
    q_dev = torch.from_numpy(q).cuda()
    u = I.make_uniforms(k + 1, seed + I.SEED_VERIFY_U)

    def step():
        a, n = kv.nav_verify(0, d, q_dev, u)
        kv.rollback(0, prefix)
        return a, n

    for _ in range(args.warmup):
        first = step()
    torch.cuda.synchronize()
    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        torch.mul(src, 1.0, out=dst)  # one elementwise kernel (not a blit): reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
    model.profile_select(args.prof)
    per_step = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        ts = time.perf_counter()
        res = step()  # synchronises the stream: the decision is on the host when it returns
        per_step.append(time.perf_counter() - ts)
        assert res == first, "the pass is not reproducible"
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    each_us = model.profile_read_each()
    n_launch, kern_ms = len(each_us), sum(each_us) / 1e3
    model.profile_select("off")
    # the same steps without event bracketing, to show what the events cost
    per_step_plain = []
    t1 = time.perf_counter()
    for _ in range(args.steps):
        ts = time.perf_counter()
        step()
        per_step_plain.append(time.perf_counter() - ts)
    torch.cuda.synchronize()
    elapsed_plain = time.perf_counter() - t1

    t_pass = min(elapsed, elapsed_plain) / args.steps
    alg_bytes = shape.algorithmic_bytes(prefix, k)
    esz = 4 if shape.dtype == I.DTYPE_F32 else 2
    gemm_bytes = shape.n_params_streamed() * esz  # what the GEMM launches of one pass must read
    launches_per_pass = n_launch / args.steps if args.steps else 0
    roof = None
    if n_launch:
        per_launch_bytes = gemm_bytes / launches_per_pass
        avg_ms = kern_ms / n_launch
        achieved = per_launch_bytes / (avg_ms * 1e-3) / 1e9
        all_gemm = {"achieved": achieved, "frac": achieved / HBM_PEAK_GBPS, "launches_per_pass": launches_per_pass,
                    "avg_launch_us": avg_ms * 1e3, "algorithmic_bytes_per_launch": per_launch_bytes}
        roof = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBPS, "traffic": None,
                "kernel": "gemm_bf16_kernel (all weight-streaming GEMMs of the pass)" if esz == 2 else "gemm_f32_kernel",
                **{k_: v_ for k_, v_ in all_gemm.items() if k_ not in ("achieved", "frac")}}
        per_pass = 4 * shape.n_layers + 1
        if esz == 2 and args.prof == "all_gemm" and n_launch == per_pass * args.steps:
            # every projection is a kernel of its own (the epilogue is a template parameter): the
            # roofline object is for the one the pass spends most of its time in; all five are listed
            qd, kvd, d_, F_ = shape.q_dim, shape.kv_dim, shape.d_model, shape.d_ffn
            proj = [("qkv", "gemm_bf16_kernel<16, true, EPI_QKV, ..>", (qd + 2 * kvd) * d_, lambda i: i < per_pass - 1 and i % 4 == 0),
                    ("o", "gemm_bf16_kernel<16, true, EPI_RESID, P1>", d_ * qd, lambda i: i < per_pass - 1 and i % 4 == 1),
                    ("gate_up", "gemm_bf16_kernel<16, true, EPI_SWIGLU, ..>", 2 * F_ * d_, lambda i: i < per_pass - 1 and i % 4 == 2),
                    ("down", "gemm_bf16_kernel<16, true, EPI_RESID, phases>", d_ * F_, lambda i: i < per_pass - 1 and i % 4 == 3),
                    ("lm_head", "gemm_bf16_kernel<16, true, EPI_STORE, ..>", shape.vocab * d_, lambda i: i == per_pass - 1)]
            table = {}
            for name, kname, elems, sel in proj:
                us = [t for j, t in enumerate(each_us) if sel(j % per_pass)]
                mean_us = sum(us) / len(us)
                gbps = elems * esz / (mean_us * 1e-6) / 1e9
                table[name] = {"kernel": kname, "launches_per_pass": len(us) / args.steps, "avg_launch_us": mean_us,
                               "algorithmic_bytes_per_launch": elems * esz, "achieved": gbps, "frac": gbps / HBM_PEAK_GBPS,
                               "us_per_pass": sum(us) / args.steps}
            dom = max(table, key=lambda n: table[n]["us_per_pass"])
            t_dom = table[dom]
            roof = {"bound": "hbm", "achieved": t_dom["achieved"], "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": t_dom["frac"],
                    "traffic": committed_traffic(args.workload, dom) if args.layers is None else None,
                    "kernel": t_dom["kernel"] + f" ({dom} projection: the kernel the pass spends most of its time in)",
                    "launches_per_pass": t_dom["launches_per_pass"], "avg_launch_us": t_dom["avg_launch_us"],
                    "algorithmic_bytes_per_launch": t_dom["algorithmic_bytes_per_launch"],
                    "per_projection": table, "all_weight_streaming_gemms": all_gemm}

    out = {
        "metric": "verified_tokens_per_sec", "value": k / t_pass, "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": t_pass * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if esz == 2 else "f32", "data": "synthetic",
        "config": {"workload": f"{shape.name}: NAV pass, prefix {prefix}, k={k}, batch 1, paged KV (16-token blocks)",
                   "rows_per_pass": k + 1, "accepted_len": first[0]},
        "committed_tokens_per_sec": (first[0] + 1) / t_pass,
        "hbm_algorithmic_gbps": alg_bytes / t_pass / 1e9, "hbm_frac_of_peak": alg_bytes / t_pass / 1e9 / HBM_PEAK_GBPS,
        "algorithmic_bytes_per_pass": alg_bytes,
        "ms_per_step_with_events": elapsed / args.steps * 1e3, "ms_per_step_plain": elapsed_plain / args.steps * 1e3,
        "ms_per_step_median_p10_p90": [float(np.percentile(per_step_plain, q)) * 1e3 for q in (50, 10, 90)],
        "ms_per_step_with_events_median_p10_p90": [float(np.percentile(per_step, q)) * 1e3 for q in (50, 10, 90)],
        "roofline": roof,
    }
    if not args.no_cpu_baseline:
        t0 = time.time()
        out["cpu_baseline"] = cpu_baseline(wl["shape"], weights, prefix, k, min(args.cpu_layers, shape.n_layers))
        log(f"[bench] cpu baseline took {time.time() - t0:.1f}s")
    if not args.no_extra and args.workload == "llama-8b" and args.layers is None and args.k is None and args.prefix is None:
        out["extra_configs"] = extra_configs(np, torch, I, nav, model, kv, shape, seed, prefix, sigma)
    print(json.dumps(out), flush=True)


def extra_configs(np, torch, I, nav, model8, kv8, shape8, seed8, prefix8, sigma8):
    """The other workloads of the configuration list, measured in the same run (each one guarded:
    a failure is reported in its place and never costs the headline line)."""
    extra = {}

    def guarded(name, fn):
        t0 = time.time()
        try:
            extra[name] = fn()
        except Exception as e:  # noqa: BLE001
            extra[name] = {"error": f"{type(e).__name__}: {e}"}
        log(f"[bench] extra config {name} took {time.time() - t0:.1f}s")

    # the k sweep of the 8B workload on the resident model and cache
    for kk in (1, 4, 16):
        guarded(f"llama-8b prefix {prefix8} k={kk} batch 1",
                lambda kk=kk: single_client_record(np, torch, I, nav, model8, shape8, seed8, prefix8, kk, sigma8, 20, 20, kv=kv8))
    # the same pass in two halves (pipesd_nav_verify_begin / _end): how long the call that enqueues
    # the pass keeps the host, of the whole round
    def two_halves():
        k = 8
        d, q = I.make_noisy_target_drafts(lambda ds: kv8.forward_logits(0, ds)[-1], k, shape8.vocab, sigma8,
                                          seed8 + I.SEED_NOISE + k, seed8 + I.SEED_DRAFT_U + k)
        q_dev = torch.from_numpy(q).cuda()
        u = I.make_uniforms(k + 1, seed8 + I.SEED_VERIFY_U + k)
        begin_s, total_s = [], []
        for r in range(40):
            t0 = time.perf_counter()
            kv8.nav_verify_begin(0, d, q_dev, u)
            t1 = time.perf_counter()
            kv8.nav_verify_end()
            t2 = time.perf_counter()
            kv8.rollback(0, prefix8)
            if r >= 20:
                begin_s.append(t1 - t0)
                total_s.append(t2 - t0)
        tb, tt = sum(begin_s) / len(begin_s), sum(total_s) / len(total_s)
        return {"ms_per_pass": tt * 1e3, "ms_until_begin_returns": tb * 1e3, "host_free_fraction": 1.0 - tb / tt,
                "verified_tokens_per_sec": k / tt, "passes": len(total_s)}
    guarded(f"llama-8b prefix {prefix8} k=8 batch 1, verify in two halves (begin / end)", two_halves)
    # 16 clients on the 8B model: prefixes U[256,4096], k U[1,16] redrawn every round, noisy-target
    # drafts, 50 consecutive rounds over sequences that grow
    def cfg4():
        rng = np.random.default_rng(seed8 + 1000 + I.SEED_LENGTHS)
        lens = [int(x) for x in rng.integers(256, 4097, 16)]
        ks_all = rng.integers(1, 17, (52, 16))
        return run_batched(np, torch, I, nav, model8, shape8, seed8 + 1000, lens, 50, 2, sigma8,
                           lambda r, s: int(ks_all[r, s]))
    guarded("llama-8b 16 clients, prefixes U[256,4096], k U[1,16], 50 growing rounds, sigma 0.5", cfg4)
    kv8.close()
    model8.close()
    torch.cuda.empty_cache()
    for name, steps in (("llama-1b", 50), ("tiny", 50)):
        def small(name=name, steps=steps):
            wl = I.WORKLOADS[name]
            w = I.make_weights(wl["shape"], wl["seed"] + I.SEED_WEIGHTS, threads=min(16, os.cpu_count() or 8))
            m = nav.Model(wl["shape"], w)
            try:
                return single_client_record(np, torch, I, nav, m, wl["shape"], wl["seed"], wl["prefix"], wl["k"], wl["sigma"],
                                            steps, 10)
            finally:
                m.close()
        wl = I.WORKLOADS[name]
        guarded(f"{name} prefix {wl['prefix']} k={wl['k']} batch 1", small)
    # the long-context 13B workload: 4 clients, prefix 8192, k = 16, sigma 1.0, through the batched call
    def cfg5():
        wl = I.WORKLOADS["llama-13b"]
        w = I.make_weights(wl["shape"], wl["seed"] + I.SEED_WEIGHTS, threads=min(16, os.cpu_count() or 8))
        m = nav.Model(wl["shape"], w)
        del w
        try:
            return run_batched(np, torch, I, nav, m, wl["shape"], wl["seed"] + 1000, [wl["prefix"]] * 4, 8, 2, wl["sigma"],
                               lambda r, s: wl["k"])
        finally:
            m.close()
    guarded("llama-13b 4 clients, prefix 8192, k=16, sigma 1.0, growing rounds", cfg5)
    return extra


if __name__ == "__main__":
    main()
