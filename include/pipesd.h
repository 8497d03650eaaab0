/*
 * pipesd.h — C ABI of the MI355X (gfx950) implementation of the cloud-side hot path of PipeSD:
 * the target model's non-autoregressive verification (NAV) pass.
 *
 * What one pass computes (Sec. 2.2 "speculative round", Sec. 2.3, Sec. 4.2 "Target Model",
 * Appendix B): the cloud holds the committed text of a client; the edge sends k draft tokens;
 * the target model runs ONE causal forward over them on top of its cached prefix, accepts the
 * drafts that pass the speculative-sampling test, replaces the first rejected one by a corrected
 * token (or, if all k pass, contributes one extra token), and drops the rejected suffix so that
 * drafting can restart from the last accepted token.
 *
 * Sequence state between passes: committed tokens t_0..t_{n-1} (n = "prefix length"); keys and
 * values cached for t_0..t_{n-2}; t_{n-1} is PENDING (it is the previous pass's corrected/extra
 * token, or the last prompt token, and has not been through the model).  A pass therefore runs
 * m = k + 1 rows: [pending, d_1..d_k] at positions n-1 .. n-1+k.  Row i-1 yields the target
 * distribution p_i that judges draft i; row k yields the extra-token distribution p_{k+1}.
 *
 * Conventions
 *   - every function returns PIPESD_OK (0) or a negative pipesd_status; nothing throws or aborts;
 *   - a call that fails changes no state of its handles;
 *   - "device" pointers are HIP device memory on the current device, "host" pointers are ordinary
 *     host memory; `stream` is a hipStream_t passed as void* (NULL = the null stream);
 *   - handles are owned by the library; buffers passed in are borrowed only for the duration
 *     stated at each function;
 *   - calls on one handle are not thread-safe and calls that share a model overlap on the GPU only
 *     if issued on the same stream (they share the model's activation workspace).
 */
#ifndef PIPESD_H
#define PIPESD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  PIPESD_OK = 0,
  PIPESD_EINVAL = -1, /* null pointer, size or id out of range, unsupported shape */
  PIPESD_ENOMEM = -2, /* KV pool has too few free blocks, or a device allocation failed */
  PIPESD_ESTATE = -3, /* prefix_len differs from the stored length, rollback above it, verify before prefill */
  PIPESD_EHIP = -4    /* a HIP runtime call failed (including: no GPU present) */
} pipesd_status;

enum { PIPESD_F32 = 0, PIPESD_BF16 = 1 };

/* rows one pass can carry (pending + drafts), hence k <= PIPESD_MAX_ROWS - 1 */
enum { PIPESD_MAX_ROWS = 32 };

/* Decoder-only transformer (Sec. 2.1) in the Llama form: RMSNorm before attention and before the
 * feed-forward block, rotary positions on element pairs (i, i + head_dim/2) with angle
 * pos * rope_base^(-2i/head_dim), grouped-query attention (query head g reads KV head
 * g / (n_q_heads / n_kv_heads)), SwiGLU feed-forward, no biases, untied LM head.
 * dtype selects the storage type of all matrices and of the KV cache; norm gains are fp32. */
typedef struct {
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
  float rms_eps, rope_base;
  int32_t dtype; /* PIPESD_F32 or PIPESD_BF16 */
} pipesd_config;

/* Device pointers to the caller's weights, every matrix [out][in] row-major in `dtype`.
 * Arrays of per-layer pointers are host arrays of n_layers device pointers. */
typedef struct {
  const void *tok_emb;         /* [vocab][d_model] */
  const void *final_norm;      /* [d_model] fp32 */
  const void *lm_head;         /* [vocab][d_model] */
  const void *const *attn_norm; /* [d_model] fp32 each */
  const void *const *ffn_norm;  /* [d_model] fp32 each */
  const void *const *wq;        /* [n_q_heads*head_dim][d_model] */
  const void *const *wk;        /* [n_kv_heads*head_dim][d_model] */
  const void *const *wv;        /* [n_kv_heads*head_dim][d_model] */
  const void *const *wo;        /* [d_model][n_q_heads*head_dim] */
  const void *const *w_gate;    /* [d_ffn][d_model] */
  const void *const *w_up;      /* [d_ffn][d_model] */
  const void *const *w_down;    /* [d_model][d_ffn] */
} pipesd_weights;

typedef struct pipesd_model pipesd_model;
typedef struct pipesd_kv pipesd_kv;

/* Target model handle (Sec. 4.2: the cloud keeps one target model for all clients, Appendix I).
 * The weights are re-tiled into library-owned device memory in the order the matrix cores read
 * them, synchronously: when the call returns the caller may free its own copies.
 * weights == NULL creates a shape-only handle without device memory (for planning KV pools and
 * exercising the bookkeeping without a GPU); compute calls on it return PIPESD_ESTATE.
 * EINVAL: null cfg/out, non-positive sizes, n_q_heads not a multiple of n_kv_heads, odd head_dim,
 * head_dim > 128, or (bf16) d_model, n_q_heads*head_dim or d_ffn not a multiple of 512,
 * head_dim other than 64 or 128, or d_model above 8192. */
int pipesd_model_create(const pipesd_config *cfg, const pipesd_weights *weights, pipesd_model **out);
int pipesd_model_destroy(pipesd_model *model);

/* Bytes of one KV block: block_tokens tokens x all layers x (K and V) x n_kv_heads x head_dim. */
size_t pipesd_kv_block_bytes(const pipesd_model *model, int32_t block_tokens);

/* Paged KV cache for up to max_seqs clients over a caller-allocated device pool (borrowed until
 * pipesd_kv_destroy).  The pool holds floor(pool_bytes / block_bytes) blocks of block_tokens
 * (16) tokens; per layer the keys of a block are [kv_head][token][head_dim] and the values
 * [kv_head][head_dim][token].  pool == NULL gives bookkeeping only (see pipesd_model_create).
 * With a pool, the model's scratch for attention partials is sized here for the largest pass this
 * pool admits (about 0.5 MB per 256 pool tokens for 32 query heads of 128), so that no verify call
 * allocates.
 * EINVAL: block_tokens != 16, max_seqs < 1, pool too small for one block, pool not 256-byte aligned;
 * ENOMEM: the block tables or the scratch cannot be allocated. */
int pipesd_kv_create(const pipesd_model *model, int32_t max_seqs, int32_t block_tokens, void *pool,
                     size_t pool_bytes, pipesd_kv **out);
int pipesd_kv_destroy(pipesd_kv *kv);

/* Forget client `seq`: length 0, all its blocks back to the pool. */
int pipesd_seq_reset(pipesd_kv *kv, int32_t seq);

/* Commit n more tokens (host array) to client `seq`: afterwards keys/values are cached for all
 * committed tokens but the last, which is pending.  Runs the same forward as a verify pass in row
 * blocks (128 rows on a bf16 model, 32 on an fp32 one), without the LM head.  Returns after the work is enqueued on `stream`.
 * ENOMEM if the pool cannot hold the new rows. */
int pipesd_prefill(pipesd_model *model, pipesd_kv *kv, int32_t seq, const int32_t *tokens, int32_t n,
                   void *stream);

/* One NAV pass for one client (Sec. 2.2; Appendix B).
 *   prefix_len    committed length the caller believes the client has (ESTATE if it differs);
 *   draft_tokens  host [k], 1 <= k <= PIPESD_MAX_ROWS - 1;
 *   draft_probs   device fp32 [k][vocab]: the draft model's full distribution q_i at each draft
 *                 position; NULL selects token matching (accept d_i iff it is the target's argmax,
 *                 lowest index on ties; next = argmax);
 *   uniforms      host [k+1] in [0,1): u_1..u_k for the tests, u_{k+1} for the one draw (ignored
 *                 when draft_probs is NULL, may then be NULL).
 * Rule: accept d_i iff u_i < min(1, p_i(d_i) / q_i(d_i)) (fp32 division; 0/0 rejects), stopping at
 * the first rejection; accepted_len = a.  next_token is drawn from max(0, p_{a+1} - q_{a+1}) if
 * a < k, else from p_{k+1}, by the integer inverse CDF: weights floor(w * 2^40) summed as 64-bit
 * integers to W, threshold T = floor(u * 2^24) * W >> 24, result the smallest j whose running sum
 * exceeds T (W = 0: lowest-index argmax of p_{a+1}).
 * Afterwards the client's committed length is prefix_len + a + 1 with next_token pending, the
 * cache keeps the pending row and the a accepted rows, the k - a rejected rows are zeroed and
 * blocks wholly beyond the kept rows return to the pool.  Synchronises `stream`; the two host
 * outputs are valid on return. */
int pipesd_nav_verify(pipesd_model *model, pipesd_kv *kv, int32_t seq, int32_t prefix_len,
                      const int32_t *draft_tokens, int32_t k, const float *draft_probs,
                      const float *uniforms, int32_t *accepted_len, int32_t *next_token, void *stream);

/* The same pass in two halves, for a caller that has other work while the GPU runs it (receiving the
 * next drafts, enqueueing work on other streams): pipesd_nav_verify_begin takes the arguments of
 * pipesd_nav_verify, runs all its checks, enqueues the whole pass on `stream` and returns WITHOUT
 * waiting; pipesd_nav_verify_end waits for it and does the bookkeeping, with the results and error
 * behaviour of pipesd_nav_verify (bit-identical results).  draft_tokens and uniforms are copied by
 * begin; draft_probs (device memory) must stay valid until end returns.  Between begin and end the
 * model's buffers and the pool's blocks belong to the pass: every other entry point that computes
 * with the model (prefill, verify, verify_batch, verify_chain, verify_begin, forward_logits) and
 * pipesd_kv_rollback / pipesd_seq_reset on that pool return PIPESD_ESTATE, as does end without a
 * begin.  A model must not be destroyed between begin and end.
 * pipesd_nav_verify_done sets *done to 1 once the pass has finished on the device (end will not
 * block), else 0; it never waits. */
int pipesd_nav_verify_begin(pipesd_model *model, pipesd_kv *kv, int32_t seq, int32_t prefix_len,
                            const int32_t *draft_tokens, int32_t k, const float *draft_probs,
                            const float *uniforms, void *stream);
int pipesd_nav_verify_done(pipesd_model *model, int32_t *done);
int pipesd_nav_verify_end(pipesd_model *model, int32_t *accepted_len, int32_t *next_token);

/* One NAV pass for each of n_seqs clients (several edge devices verified by one cloud model,
 * Appendix I): client i = seq_ids[i] (pairwise distinct, 1 <= n_seqs <= 256) with committed length
 * prefix_lens[i] and k_per_seq[i] drafts.  draft_tokens_concat (host) holds the clients' drafts one
 * after the other, uniforms_concat (host) their k_i + 1 uniforms one after the other (a client's
 * slots are skipped over but not read when it uses token matching); draft_probs_per_seq is a host
 * array of n_seqs device pointers ([k_i][vocab] fp32 each; a NULL entry, or a NULL array, selects
 * token matching).  Per client the computation, the result and the state afterwards are those of
 * pipesd_nav_verify.  All arguments and the pool's free blocks are checked before anything
 * changes: an error leaves every client as it was.  On a bf16 model the clients' rows are packed,
 * in the order given, into passes of up to 256 rows and 16 clients, so that the weights are
 * streamed once per pass and not once per client (a row's result does not depend on which rows
 * share its pass: the results are bit-identical to single calls); an fp32 model runs one pass per
 * client.  All work is enqueued on `stream`, which is synchronised once; accepted_len and
 * next_token are host arrays [n_seqs]. */
int pipesd_nav_verify_batch(pipesd_model *model, pipesd_kv *kv, int32_t n_seqs, const int32_t *seq_ids,
                            const int32_t *prefix_lens, const int32_t *k_per_seq,
                            const int32_t *draft_tokens_concat, const float *const *draft_probs_per_seq,
                            const float *uniforms_concat, int32_t *accepted_len, int32_t *next_token,
                            void *stream);

/* Cut client `seq` back to new_prefix_len committed tokens (1 <= new <= current, else ESTATE); the
 * last kept token becomes pending (Appendix B: buffered drafts that are no longer valid are
 * discarded and drafting restarts from the last accepted token).  Host bookkeeping only. */
int pipesd_kv_rollback(pipesd_kv *kv, int32_t seq, int32_t new_prefix_len);
int pipesd_kv_len(const pipesd_kv *kv, int32_t seq, int32_t *prefix_len);
/* Blocks currently free in the pool / held by a client. */
int pipesd_kv_free_blocks(const pipesd_kv *kv, int32_t *n_free);
int pipesd_kv_seq_blocks(const pipesd_kv *kv, int32_t seq, int32_t *n_blocks);

/* Test hook: run rows [pending, tokens[0..n_extra-1]] (n_extra >= 0 host tokens) through the
 * forward and copy the (n_extra + 1) x vocab fp32 logits to the host array `logits_out`.  The rows
 * are written to the cache but not committed: the client's state is unchanged.  Synchronises. */
int pipesd_forward_logits(pipesd_model *model, pipesd_kv *kv, int32_t seq, const int32_t *tokens,
                          int32_t n_extra, float *logits_out, void *stream);

/* Test hook: the decision step alone on caller-supplied probabilities.
 *   p device fp32 [k+1][vocab], q device fp32 [k][vocab], draft_tokens host [k], uniforms host [k+1].
 * Same rule and same kernels as pipesd_nav_verify.  Synchronises. */
int pipesd_spec_accept(const float *p, const float *q, const int32_t *draft_tokens, int32_t k,
                       int32_t vocab, const float *uniforms, int32_t *accepted_len, int32_t *next_token,
                       void *stream);

/* For callers that cannot allocate device memory: code recorded under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  The decision step of pipesd_spec_accept with no
 * allocation, no copy and no synchronisation: the kernels' scratch (4096 bytes: the 64 partial sums
 * of the integer CDF and the arrival counter) is a static device array inside the library, one copy
 * per GPU, held until the process ends.
 *   p, q, draft_tokens, uniforms as for pipesd_spec_accept; result_dev is DEVICE memory, int32[2]:
 *   {accepted_len, next_token}, valid once the work enqueued on `stream` has completed.
 * Limits: 1 <= k <= PIPESD_STATIC_MAX_K, 1 <= vocab <= PIPESD_STATIC_MAX_VOCAB; beyond them the call
 * returns PIPESD_EINVAL and pipesd_last_hip_error() says which limit.  Every call on a GPU uses that
 * GPU's one scratch array: calls that overlap on one GPU (two streams, two threads) race; calls on
 * one stream are ordered and safe.  The arrival counter is cleared by a small kernel at the start
 * of every call, so a graph that records this call records no memset node. */
enum { PIPESD_STATIC_MAX_K = PIPESD_MAX_ROWS - 1, PIPESD_STATIC_MAX_VOCAB = 1 << 22 };
int pipesd_spec_accept_static(const float *p, const float *q, const int32_t *draft_tokens, int32_t k,
                              int32_t vocab, const float *uniforms, int32_t *result_dev, void *stream);

/* Chained rounds on proactively sent drafts (Appendix B: while a round is being verified the edge
 * goes on drafting and sending; the cloud buffers those tokens and keeps them only if the round
 * accepts every draft AND its extra token equals the first buffered token).
 *   Round 0 is an ordinary round: k_per_round[0] drafts.  Round r >= 1 brings a buffer of
 *   1 + k_per_round[r] tokens: the edge's guess of round r-1's extra token, then round r's drafts.
 *   tokens_concat (host) holds round 0's drafts, then each buffer; draft_probs_per_round[r] (host
 *   array of device pointers, or NULL = token matching for every round; entries may be NULL) is the
 *   fp32 [k_r][vocab] distribution block of round r's DRAFTS (the guess has none: it is compared with
 *   the target's own extra token); uniforms_concat (host) holds k_r + 1 values per round, one round
 *   after the other (ignored for token-matching rounds, may then be NULL).
 * Round r runs iff every earlier round ran, accepted all its drafts and produced the guessed extra
 * token; each round that runs is exactly a pipesd_nav_verify call on the state the round before
 * left.  *rounds_run (>= 1 on success) tells how many ran; accepted_len / next_token (host,
 * [n_rounds]) are filled for those.  1 <= n_rounds <= 16.
 * bf16 models: every round is enqueued at once for the state its buffer presumes, the rule above is
 * applied on the device (a small step behind each round's decision sets a word that gates the next
 * round's launches: a round whose buffer is invalid streams no weights and writes no result), and
 * the call synchronises ONCE; the host then books the rounds that ran.  fp32 models and the fused
 * layer path apply the rule on the host between single calls (one synchronisation per round).
 * Both give bit for bit what single calls give.
 * Errors: all argument checks (PIPESD_EINVAL), the state check (PIPESD_ESTATE) and the check that the
 * pool can hold the longest possible outcome (PIPESD_ENOMEM) come before anything changes.  A HIP
 * failure on the bf16 path leaves the sequence as it was before the call (*rounds_run = 0); on the
 * host-rule path a failure in round r > 0 leaves rounds 0..r-1 committed and *rounds_run = r. */
int pipesd_nav_verify_chain(pipesd_model *model, pipesd_kv *kv, int32_t seq, int32_t prefix_len,
                            int32_t n_rounds, const int32_t *k_per_round, const int32_t *tokens_concat,
                            const float *const *draft_probs_per_round, const float *uniforms_concat,
                            int32_t *accepted_len, int32_t *next_token, int32_t *rounds_run, void *stream);

/* Test hook: copy the cached key and value of one (layer, position) of client `seq` to host fp32
 * arrays [n_kv_heads*head_dim] (keys as stored, i.e. rotated).  Synchronises the device. */
int pipesd_kv_read(const pipesd_model *model, const pipesd_kv *kv, int32_t seq, int32_t layer,
                   int32_t pos, float *k_out, float *v_out);

/* Launch strategy of the layer stack.  By default every projection and every attention step is a
 * kernel launch of its own.  After pipesd_model_set_fused(model, 1) a bf16 pass of up to 16 rows
 * runs all decoder layers in ONE cooperative kernel instead (device-wide barriers between the
 * projections, weights requested ahead of each barrier); passes it does not take keep the per-
 * projection launches.  Both run the same device code on the same tiles in the same order and give
 * bit-identical results.  pipesd_model_fused_launches counts the fused launches so far.
 * PIPESD_PROF_GEMM_* classes time nothing while the fused kernel is in use (PIPESD_PROF_LAYERS does). */
int pipesd_model_set_fused(pipesd_model *model, int32_t on);
int pipesd_model_fused_launches(const pipesd_model *model, int64_t *n);

/* GEMM kernel of bf16 passes of more than 64 rows (batched verification, prompt ingestion).  Two
 * kernels compute them: the narrow one of the single-client pass, run by groups of workgroups that
 * share the weights through a chiplet's L2, and a wide one that stages the activations of all rows
 * in LDS.  mode 0 (default): per product, whichever was measured faster for its shape; 1: always the
 * narrow kernel; 2: always the wide one.  Both accumulate every output in the same order and give
 * bit-identical results, so the mode changes speed only.  PIPESD_EINVAL for another mode. */
int pipesd_model_set_wide_gemm(pipesd_model *model, int32_t mode);

/* Per-kernel timing for roofline accounting: when enabled, every launch of the selected kernel
 * class is timed with HIP events on its stream (the bf16 GEMM launches carry their own start and
 * stop events, the other classes are bracketed by recorded events).  pipesd_profile_read waits for them and returns
 * the number of launches and their summed duration since the last read. */
enum { PIPESD_PROF_OFF = 0, PIPESD_PROF_GEMM_QKV = 1, PIPESD_PROF_GEMM_O = 2, PIPESD_PROF_GEMM_GATEUP = 3,
       PIPESD_PROF_GEMM_DOWN = 4, PIPESD_PROF_GEMM_LMHEAD = 5, PIPESD_PROF_ATTN = 6, PIPESD_PROF_VERIFY = 7,
       PIPESD_PROF_ALL_GEMM = 8, PIPESD_PROF_LAYERS = 9 };
int pipesd_profile_select(pipesd_model *model, int32_t kernel_class);
int pipesd_profile_read(pipesd_model *model, int32_t *n_launches, double *total_ms);
/* The same, launch by launch: copies the durations (microseconds, in launch order) of the timed
 * launches since the last read into host array us_out (at most `cap` values) and sets *n_launches
 * to their number.  With PIPESD_PROF_ALL_GEMM a bf16 pass yields QKV, O, gate/up, down per layer,
 * then the LM head. */
int pipesd_profile_read_each(pipesd_model *model, double *us_out, int32_t cap, int32_t *n_launches);
/* While PIPESD_PROF_LAYERS is selected the fused layer kernel also records a device clock at the
 * start of each of its 4*n_layers steps (QKV + attention, O, gate/up, down per layer).  Copies the
 * step durations of the most recent fused launch, in microseconds, into host array us_out (at most
 * `cap` values) and sets *n_steps to 4*n_layers (0 if no fused launch was recorded).  Synchronises
 * the device. */
int pipesd_profile_read_steps(pipesd_model *model, double *us_out, int32_t cap, int32_t *n_steps);

/* ---- Edge-side scheduling of a speculative round: host arithmetic only, no GPU work ----------
 *
 * Token batching (Sec. 3.2).  The N draft tokens of a round leave the edge in K batches; B =
 * (b_1..b_K), 1 = b_1 < .. < b_K <= N, holds the 1-based index of each batch's first token
 * (Eq. (1)).  Generating one token takes gamma; sending a batch of n tokens takes alpha + beta n
 * (Eqs. (2), (3)); a batch goes on the link when it has been generated and the batch before it has
 * been delivered (Eqs. (4), (5)).  All times in one unit of the caller's choice, fp64, >= 0.
 *
 * pipesd_batching_time: *time_out = T of Eq. (6), from the start of generation to the delivery of
 * the last batch, for the batching `first` (host, n_batches entries).  PIPESD_EINVAL: null
 * pointer, n_tokens < 1, a sequence that breaks Eq. (1), a negative or non-finite cost. */
int pipesd_batching_time(int32_t n_tokens, const int32_t *first, int32_t n_batches, double alpha,
                         double beta, double gamma, double *time_out);

/* The batching of minimal T for a scheduling window of n_tokens tokens (Sec. 4.1, Algorithm 1;
 * optimal by Theorem 1).  Writes the K first-token indices to first_out (host, room for n_tokens
 * entries), K to *n_batches_out and the minimal T to *time_out; pipesd_batching_time of the
 * returned batching gives the same T bit for bit.  Where several batchings reach the minimum, the
 * one whose last batch is longest is returned (and so on towards the front).  Quadratic in n_tokens:
 * PIPESD_EINVAL above 16384 tokens, for a null pointer, n_tokens < 1, a negative or non-finite
 * cost; PIPESD_ENOMEM if the tables cannot be allocated. */
int pipesd_batching_optimal(int32_t n_tokens, double alpha, double beta, double gamma,
                            int32_t *first_out, int32_t *n_batches_out, double *time_out);

/* Dual-threshold NAV trigger (Sec. 3.3) over a stream of draft-token confidences P(D_1), P(D_2), ..
 * (host, n values in [0, 1]).  C_1 is the product of the confidences drafted since the last NAV;
 * token n ends the round when C_1 P(D_n) <= r1 or P(D_n) <= r2, and C_1 returns to 1 after either
 * (the token that fires belongs to the round it ends).  max_len >= 1 also ends a round that has
 * reached the longest draft one verification pass takes (not in the paper; pass a value above n to
 * switch it off).  Writes the draft length of every complete round to lengths_out (host, room for
 * lengths_cap entries; the walk stops in front of a round that does not fit), their number to
 * *n_rounds_out and the number of confidences those rounds cover to *consumed_out: the tokens
 * after them have not fired yet.  PIPESD_EINVAL: null pointer, negative size, max_len < 1, a
 * threshold or confidence outside [0, 1] (NaN included). */
int pipesd_trigger_rounds(const double *confidence, int64_t n, double r1, double r2, int32_t max_len,
                          int32_t *lengths_out, int64_t lengths_cap, int64_t *n_rounds_out,
                          int64_t *consumed_out);

/* ---- Autotuner of the trigger thresholds (Sec. 3.3 "BO autotuner"; appendix "Design and
 * Performance Evaluation of BO"): host arithmetic only, no GPU work ------------------------------
 *
 * The thresholds (R1, R2) in (0,1)^2 are tuned by Bayesian optimisation of the measured time per
 * accepted token (to be MINIMISED): Gaussian-process regression with a Matern kernel, Expected
 * Improvement with exploration parameter xi (0.1 in the paper), one random initial sample, 16
 * samples in all, each the mean over 20 accepted tokens.  The caller owns the loop and the
 * measurements: it keeps the samples x (host, n pairs (R1, R2), row-major) and their measured values
 * y (host, n), and asks for the next pair to try.  Fixed beyond what the paper names: Matern
 * smoothness 5/2 with length scale `length_scale` on the Euclidean distance and unit variance,
 * `noise` >= 0 added to the diagonal, observations standardised (zero mean, unit population
 * standard deviation; scale 1 if they are all equal), no hyper-parameter fit, fp64.
 *
 * pipesd_bo_posterior (test hook and building block): posterior mean and standard deviation, in the
 * units of y, at m query points q (host, m pairs) into mean_out / std_out (host, m).
 * pipesd_bo_suggest: the maximiser of EI over the midpoints ((i + 0.5) / grid, (j + 0.5) / grid) of a
 * uniform grid x grid raster (the first in raster order, R1 slowest, among equal values) into
 * next_out (host, 2), and its EI on the standardised scale into *ei_out (may be NULL).
 * EI = I Phi(I / s) + s phi(I / s) with I = min(y_s) - mu_s - xi; max(I, 0) where s = 0.
 * PIPESD_EINVAL: null pointer, n < 1 or n > 4096, grid < 1 or > 1024, non-finite values, length_scale
 * <= 0, negative noise or xi, or a kernel matrix that is not positive definite (the same point
 * twice with noise 0); PIPESD_ENOMEM if the tables cannot be allocated. */
int pipesd_bo_posterior(const double *x, const double *y, int32_t n, double length_scale, double noise,
                        const double *q, int32_t m, double *mean_out, double *std_out);
int pipesd_bo_suggest(const double *x, const double *y, int32_t n, double length_scale, double noise,
                      double xi, int32_t grid, double *next_out, double *ei_out);

const char *pipesd_strerror(int status);
/* Text of the HIP call that made this thread's most recent call return PIPESD_EHIP ("" if none). */
const char *pipesd_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* PIPESD_H */
