"""CPU checker for the NAV pass: TEST INFRASTRUCTURE, not part of the product.

A plain, slow numpy implementation of what the cloud side of PipeSD computes in one
speculative round (Sec. 2.2; Appendix B): one causal forward of a decoder-only target
model over [pending token, d_1..d_k] on top of a cached prefix, the speculative-sampling
accept / correct / extra-token decision, and the rollback of the rejected suffix.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this package.
It shares no code with the HIP library and imports nothing from it; inputs arrive as plain
numpy arrays.

Precision: fp32 arrays throughout (weights stored as bf16 are widened exactly), which is the
precision the decision step is defined in; matmuls are numpy's.  The KV cache is part of the
state's definition: a bf16 model keeps its keys and values in bf16, so the checker rounds them
on append exactly as any bf16 cache must, and reads the rounded values.  OracleModel(...,
kv_format="fp32") switches that rounding off: the checker is then fp32 throughout, and the GPU
tests report the bf16 path's distance from it as well.

Pins (tests/test_oracle_*.py): row block == sequential single-token forwards; greedy ==
longest argmax-matching prefix; exact output law == target law on tiny vocabularies, measured
by bisection on the real decision function; acceptance probability == sum min(p, q); special
cases; an independent re-statement of the forward with torch primitives; a hand-computed
two-token example; Table 7's accounting of a + 1 committed tokens per pass; rollback
reproducibility.  The values of the logits of the seeded random models are fixed by nothing
in the paper: beyond those pins they are "parity unpinned".
"""
