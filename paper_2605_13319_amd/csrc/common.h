// Shared declarations of the NAV library's HIP sources (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/pipesd.h"

namespace pipesd {

constexpr int kMaxRows = PIPESD_MAX_ROWS;  // rows of one client per pass (k + 1)
constexpr int kMaxPassRows = 256;          // rows of all clients that share a pass (bf16)
constexpr int kBlockTokens = 16;           // tokens per KV block
constexpr int kWave = 64;

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
// float -> bf16, round to nearest even: the hardware conversion (checked on MI355X against
// add-0x7FFF-plus-lsb-and-shift on every finite float: identical)
typedef __attribute__((ext_vector_type(2))) float cvt_f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 cvt_bf16x2;
__device__ __forceinline__ uint32_t pack2_bf16(float a, float b) {  // a in the low half
  return __builtin_bit_cast(uint32_t, __builtin_convertvector((cvt_f32x2){a, b}, cvt_bf16x2));
}
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) { return (uint16_t)pack2_bf16(f, 0.f); }
// (a, b) = hi + lo with hi = bf16(x), lo = bf16(x - hi): 16 significand bits of x
__device__ __forceinline__ void split2_bf16(float a, float b, uint32_t& hi, uint32_t& lo) {
  hi = pack2_bf16(a, b);
  lo = pack2_bf16(a - __uint_as_float(hi << 16), b - __uint_as_float(hi & 0xffff0000u));
}
__device__ __forceinline__ float load_elem(const float* p, size_t i) { return p[i]; }
__device__ __forceinline__ float load_elem(const uint16_t* p, size_t i) { return bf16_bits_to_f32(p[i]); }
__device__ __forceinline__ void store_elem(float* p, size_t i, float v) { p[i] = v; }
__device__ __forceinline__ void store_elem(uint16_t* p, size_t i, float v) { p[i] = f32_to_bf16_bits(v); }

// Where a sequence's keys and values live.  Per layer the pool holds all key blocks, then all
// value blocks; a key block is [kv_head][token][head_dim], a value block [kv_head][head_dim][token].
struct KvView {
  void* pool;
  const int32_t* table;  // device block table of the sequence
  int64_t layer_stride;  // elements between layers (2 * n_blocks * block_elems)
  int64_t v_offset;      // elements from a layer's key blocks to its value blocks
  int32_t block_elems;   // n_kv_heads * 16 * head_dim
  int32_t n_kv_heads, head_dim;
};

// Rows of several clients in one pass (bf16 path): where each row sits in its own client's sequence.
struct RowMap {
  int32_t pos[kMaxPassRows];        // position of the row in its client's sequence
  int32_t table_off[kMaxPassRows];  // entries from KvView::table to the client's block table
};
constexpr int kMaxPassClients = 16;  // clients whose rows share one pass (each has at least 2 rows)
struct AttnClient {
  int32_t row_off, m, start_pos;  // the client's rows in the pass; position of its first row
  int32_t table_off;              // entries from KvView::table to the client's block table
  int32_t nsplit, part_off;       // splits of its context; floats from the partial buffer's start to the client's partials
  int32_t span, count_off;        // streaming kernel: tokens per split, the client's first arrival counter
};
struct AttnBatch {
  int32_t n;
  AttnClient c[kMaxPassClients];
};

__device__ __forceinline__ int64_t k_index(const KvView& kv, int layer, int pos, int kvh, int e) {
  const int blk = kv.table[pos / kBlockTokens];
  return (int64_t)layer * kv.layer_stride + (int64_t)blk * kv.block_elems +
         ((int64_t)kvh * kBlockTokens + (pos % kBlockTokens)) * kv.head_dim + e;
}
__device__ __forceinline__ int64_t v_index(const KvView& kv, int layer, int pos, int kvh, int e) {
  const int blk = kv.table[pos / kBlockTokens];
  return (int64_t)layer * kv.layer_stride + kv.v_offset + (int64_t)blk * kv.block_elems +
         ((int64_t)kvh * kv.head_dim + e) * kBlockTokens + (pos % kBlockTokens);
}

// ActPack: activations handed from one kernel to the next GEMM, already in the B-operand layout of
// the 16x16x32 bf16 MFMA and split into a bf16 hi + lo pair.  For a consumer with K columns the
// buffer is uint4[K/32][nt row tiles][hi, lo][64 entries] (nt = 2 for passes of up to 32 rows, 8 for
// the largest passes of several clients): entry (c, g) of k-step ks holds columns ks*32 + g*8 .. +7
// of row (row tile)*16 + c and is what MFMA lane g*16 + c consumes.  Within a 1 KB fragment:
//  * nt = 2: entry c*4 + g.  A row's 64 bytes are contiguous, so a pass with m < 16 rows (the usual
//    single-client pass) touches only the first m*64 bytes of each fragment;
//  * nt = 8: entry g*16 + c, the consumer's lane order: full tiles are read with lane l taking
//    entry l (fully coalesced, and a straight copy into LDS for the wide GEMM), and the 16 lanes of
//    an epilogue that hold the same columns of 16 rows store 256 contiguous bytes.
__device__ __forceinline__ size_t act_index(int kstep, int mt, int hl, int c, int g, int nt) {
  return (((size_t)kstep * nt + mt) * 2 + hl) * 64 + (nt == 2 ? c * 4 + g : g * 16 + c);
}
inline size_t act_pack_bytes(int K, int nt) { return (size_t)(K / 32) * nt * 2 * 64 * 16; }

// split 8 consecutive columns k0..k0+7 (k0 % 8 == 0) of `row` into hi + lo and store them
__device__ __forceinline__ void store_act8(uint4* buf, int row, int k0, const float (&v)[8], int nt) {
  uint32_t h[4], l[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) split2_bf16(v[2 * i], v[2 * i + 1], h[i], l[i]);
  const int g = (k0 & 31) >> 3, c = row & 15;
  buf[act_index(k0 >> 5, row >> 4, 0, c, g, nt)] = make_uint4(h[0], h[1], h[2], h[3]);
  buf[act_index(k0 >> 5, row >> 4, 1, c, g, nt)] = make_uint4(l[0], l[1], l[2], l[3]);
}

// ---------------------------------------------------------------------------------------------
// launchers (one per kernel family); all enqueue on `st` and return the launch status
// ---------------------------------------------------------------------------------------------
struct RowTokens {
  int32_t tok[kMaxRows];
};
struct PassTokens {
  int32_t tok[kMaxPassRows];
};

// embedding gather into the fp32 residual stream + rotary cos/sin of the m positions; for bf16
// models also the packed, gained copy and the per-row sum of squares for the first fused norm
// `map` gives every row's position; it is also copied to `map_dev` (if not null) for the kernels
// that need it per row
hipError_t launch_setup_rows(int dtype, const void* tok_emb, const PassTokens& toks, const RowMap& map, int m,
                             int d_model, int head_dim, const double* theta, float* xres, float* rope_cs,
                             const float* gain, void* xpk, int act_tiles, float* ssq_out, int ssq_stride,
                             RowMap* map_dev, hipStream_t st);

// ---- fp32 path (plain ALU kernels) ----
hipError_t launch_rmsnorm_rows(const float* x, const float* gain, float eps, int m, int d, float* out, hipStream_t st);
hipError_t launch_gemm_f32(const float* act, int lda, const float* w, int N, int K, int m, float* out, int ldo,
                           int add_to_out, hipStream_t st);
hipError_t launch_rope_append_f32(const float* qkv, int m, int start_pos, int layer, int n_q_heads, const KvView& kv,
                                  const float* rope_cs, float* qbuf, hipStream_t st);
hipError_t launch_silu_mul(const float* gu, int m, int d_ffn, float* act2, hipStream_t st);

// ---- bf16 path: skinny GEMM on the matrix cores over re-tiled weights ----
enum GemmEpilogue { EPI_STORE = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_QKV = 3 };
enum PackMode { PACK_PLAIN = 0, PACK_HALVES = 1 };

struct GemmPlan {  // launch shape of one GEMM
  int K, N, ntiles;
  int W, P, grid, tg;  // waves per workgroup, K phases per wave, workgroups, n-tiles per group
};

struct GemmCall {
  const void* wp;     // re-tiled weights [N][K]
  int N, K, m;
  const void* actp;   // packed activations (ActPack with K columns)
  int act_tiles;      // row tiles of this pass's ActPack buffers (input and output)
  const float* ssq_in;  // fused RMSNorm: [row][ssq_stride] partial sums of x^2 (ssq_parts used), or nullptr
  int ssq_parts, ssq_stride;
  float eps;
  int epi;
  float* out;         // STORE: [m][ldo] logits; RESID: new residual stream [m][ldo]; QKV: query buffer [m][ldo]
  const float* res_in;  // RESID: residual stream the product is added to (may be `out`)
  int ldo;
  void* outp;         // RESID: packed x_new * gain_next; SWIGLU: packed silu(gate)*up
  const float* gain_next;
  float* ssq_out;     // RESID: [row][ssq_stride] per-tile sums of x_new^2
  // QKV epilogue
  KvView kv;
  int layer, start_pos, n_q_heads;
  const float* rope_cs;
  const RowMap* rows;  // device; nullptr: one client, row r at position start_pos + r, table kv.table
  // passes of more than 64 rows: workspace for the running sums of K-split workgroups
  // (gemm_wide_workspace_bytes; may be null when that is 0)
  void* wide_ws = nullptr;
  size_t wide_ws_bytes = 0;
  int wide_mode = 0;  // 0: kernel chosen by shape, 1: narrow kernel, 2: wide kernel
  // optional: events that take the kernel's own start and end (no marker packets around it)
  hipEvent_t ev_start = nullptr, ev_stop = nullptr;
  // optional device word: the launch does nothing if it holds 0 (a round of a chain whose buffer
  // turned out to be invalid; narrow kernel only)
  const int32_t* gate = nullptr;
};
hipError_t launch_gemm_bf16(const GemmCall& c, hipStream_t st);
int device_cu_count();
// bytes of GemmCall::wide_ws a product with N weight rows and K columns needs on this device when
// it runs on the wide kernel (0 when that needs no workspace)
size_t gemm_wide_workspace_bytes(int N, int K);

// re-tile [rows][K] bf16 row-major (up to 3 stacked sources) into 16-row x 32-column matrix-core
// fragments; PACK_HALVES makes tile rows 8..15 the partners (second source half / second half of
// the head) of rows 0..7.
struct PackSrc {
  const uint16_t* src[3];
  int rows[3];
};
hipError_t launch_pack_bf16(const PackSrc& s, int n_src, int K, int mode, int pair_span, void* dst, int ntiles,
                            hipStream_t st);

// ---- activation buffers of the bf16 path ----
// Every tensor that one step of a pass hands to the next has its own buffer PER LAYER, so within a
// pass no address is written twice and none is read before it is written.  The per-projection
// launches do not need that; the all-layers kernel does: its workgroups may then read what other
// workgroups wrote with ordinary cached loads, because a cache can hold no older copy of a line.
// Index l = 0..n_layers-1, and n_layers for the tensors entering the LM head.
struct ActArena {
  char* base;
  size_t off_xa, off_xb, off_ap, off_gp, off_ra, off_rb, off_q, off_sa, off_sb;  // first instance of each kind
  size_t x_bytes, ap_bytes, gp_bytes, r_bytes, q_bytes, s_bytes;                // distance between layers
  float* part;          // attention partials
  size_t part_stride;   // floats between layers
  int ssq_stride;       // floats per row of a sums-of-squares buffer

  __host__ __device__ void* xa(int l) const { return base + off_xa + (size_t)l * x_bytes; }   // packed x*gain into QKV of layer l / LM head
  __host__ __device__ void* xb(int l) const { return base + off_xb + (size_t)l * x_bytes; }   // packed x*gain into gate/up
  __host__ __device__ void* ap(int l) const { return base + off_ap + (size_t)l * ap_bytes; }  // packed attention output
  __host__ __device__ void* gp(int l) const { return base + off_gp + (size_t)l * gp_bytes; }  // packed silu(gate)*up
  __host__ __device__ float* ra(int l) const { return (float*)(base + off_ra + (size_t)l * r_bytes); }  // residual entering layer l
  __host__ __device__ float* rb(int l) const { return (float*)(base + off_rb + (size_t)l * r_bytes); }  // residual after attention
  __host__ __device__ float* q(int l) const { return (float*)(base + off_q + (size_t)l * q_bytes); }    // rotated queries, bf16 hi | lo halves per row
  __host__ __device__ float* sa(int l) const { return (float*)(base + off_sa + (size_t)l * s_bytes); }  // sums of squares of ra(l)
  __host__ __device__ float* sb(int l) const { return (float*)(base + off_sb + (size_t)l * s_bytes); }  // sums of squares of rb(l)
  __host__ __device__ float* partials(int l) const { return part + (size_t)l * part_stride; }
};
// fills offsets; returns bytes.  per_layer = false: all layers share one buffer of each kind (enough
// for the per-projection launches), with `act_tiles` row tiles of 16 rows.
size_t act_arena_layout(ActArena& a, int n_layers, int d_model, int q_dim, int d_ffn, bool per_layer, int act_tiles);

// ---- all decoder layers of a pass in one cooperative kernel (bf16, up to 16 rows) ----
struct LayerSlabs {  // bf16 models: layer l of each tensor kind sits at base + l * bytes
  char *wqkv, *wo, *wgu, *wdown, *attn_norm, *ffn_norm;
  size_t qkv_bytes, o_bytes, gu_bytes, down_bytes, norm_bytes;
};
struct LayersCall {
  LayerSlabs slabs;
  const float* final_norm;
  int n_layers, m, start_pos, n_q_heads, head_dim, d_model, q_dim, d_ffn;
  float eps;
  KvView kv;
  const float* rope_cs;
  ActArena arena;
  unsigned* bar;  // >= 4 KB of device memory for the barrier counters and the error flag (last word used:
                  // bar[32 * 9]); read the flag back after the kernel
  unsigned long long* step_clock;  // optional [4 * n_layers + 1] device words: clock at the start of each step and at the end
};
bool layers_fused_supported(const LayersCall& c);
hipError_t launch_layers(const LayersCall& c, hipStream_t st);
constexpr int kLayersErrWord = 32 * 9;

// ---- attention over the paged cache (both dtypes) ----
struct AttnCall {
  int dtype;
  const float* q;  // fp32 cache: [rows][n_q_heads*head_dim]; bf16 cache: the same bytes per row holding bf16 hi halves, then lo halves
  KvView kv;
  int layer, m, start_pos, n_q_heads;  // fp32 cache: the one client's rows and first position
  int chunk;       // fp32 cache: tokens per workgroup
  float* part;     // per client [(head*m + r)*nsplit + split][head_dim + 4]
  float* out;      // fp32 cache: [m][n_q_heads*head_dim]
  void* outp;      // bf16 cache: packed output (ActPack with n_q_heads*head_dim columns)
  int act_tiles;   // bf16 cache: row tiles of outp
  AttnBatch batch; // bf16 cache: the clients of the pass
  const int32_t* gate = nullptr;  // bf16 cache: optional device word, the launches do nothing if it holds 0
  int stream_tiles = 0;           // bf16 cache: 0, or the query tiles per workgroup of the streaming kernel (batch planned by attn_stream_plan)
  unsigned* counters = nullptr;   // streaming kernel: kAttnCounters arrival counters, zero between launches
};
int attn_nsplit(int total_tokens, int chunk);
int attn_chunk_tokens(int dtype);  // tokens per workgroup of the attention kernel for this cache type
// Passes of at most kMaxRows rows per client, and prompt blocks of up to 128 rows alone in their
// pass (bf16 cache), take the streaming kernel.  Fills span,
// nsplit, part_off and count_off of every client of `b` (row_off, m, start_pos, table_off given) and
// returns the query tiles per workgroup, or 0 if the pass does not fit (then the split kernels run);
// *part_floats = size of the partial buffer the launch needs.  A client's split depends on its own
// context only, so its results do not depend on who shares the pass.
constexpr int kAttnCounters = kMaxPassClients * 512;
int attn_stream_plan(int n_q_heads, int n_kv_heads, int head_dim, AttnBatch& b, size_t* part_floats);
hipError_t launch_attention(const AttnCall& c, hipStream_t st);

// ---- vocabulary-wide decision ----
struct VerifyCall {
  float* logits_or_p;   // [k+1][V]
  bool from_logits;     // launch_spec_accept: logits_or_p holds logits and row_stats their softmax partials
  const float* q;       // [k][V] or nullptr (token matching)
  int k, V;
  RowTokens drafts;     // tok[0..k-1]
  float u[kMaxRows];    // u[0..k]
  float* row_stats;     // scratch [rows][nchunk][2]
  unsigned long long* scan_partial;  // scratch [nblocks]
  unsigned* counter;    // one zeroed counter
  int32_t* result;      // device [2]: accepted_len, next_token
  int32_t* result_copy; // optional second place for the two values (pinned host memory the device can write), or nullptr
};
// all clients of a pass at once (sampling rule)
struct DecisionClient {
  const float* q;       // draft distributions [k][V] (never null: token-matching clients are not part of the batch)
  int32_t row_off, k;   // the client's logits rows are row_off .. row_off + k of the pass
  int32_t slot;         // its decision goes to result[2 slot], result[2 slot + 1]
};
struct DecisionBatch {
  int32_t n;
  DecisionClient c[kMaxPassClients];
  PassTokens drafts;        // tok[row_off + j] = draft j of the client, j < k
  float u[kMaxPassRows];    // u[row_off + j] = uniform j of the client, j <= k
};
struct DecisionCall {
  const float* logits;  // [rows][V]
  int rows, V;
  DecisionBatch batch;
  float* row_stats;                  // scratch [rows][64][2]
  unsigned long long* scan_partial;  // scratch [clients][64]
  unsigned* counter;                 // [clients] zeroed counters
  int32_t* result;                   // device [slots][2]
  int32_t* result_copy;              // pinned host [slots][2], or nullptr
};
hipError_t launch_spec_accept_batch(const DecisionCall& c, hipStream_t st);
// cache trim of several clients of a pass (result[2 slot] = accepted length of the client)
struct TrimClient {
  int32_t table_off, first_pos, k, slot;
};
struct TrimBatch {
  int32_t n;
  TrimClient c[kMaxPassClients];
};
hipError_t launch_kv_trim_batch(int dtype, const KvView& kv, int n_layers, const TrimBatch& b, const int32_t* result,
                                hipStream_t st);
hipError_t launch_softmax_stats(const VerifyCall& c, hipStream_t st);  // per-row (max, sum of exp) partials of the logits
hipError_t launch_spec_accept(const VerifyCall& c, hipStream_t st);    // decision on probabilities, or (from_logits) on
                                                                        // logits + the partials of launch_softmax_stats
hipError_t launch_greedy_accept(const VerifyCall& c, hipStream_t st); // decision on logits

// zero the cached rows of positions [first_pos + result[0] + 1, first_pos + k] in every layer
hipError_t launch_kv_trim(int dtype, const KvView& kv, int n_layers, int first_pos, int k, const int32_t* result,
                          hipStream_t st);

hipError_t launch_set_table(int32_t* table, int first, const int32_t* entries, int n, hipStream_t st);
// One step of a chain of rounds on proactively sent drafts: if the round was not alive (alive_in
// holds 0; nullptr = alive), its decision is replaced by (-1, -1); alive_out (if not null) tells
// whether the next round's buffer is valid: this round alive, all k drafts accepted and the extra
// token equal to `guess`.
hipError_t launch_chain_step(int32_t* result, int32_t* result_copy, int k, int guess, const int32_t* alive_in,
                             int32_t* alive_out, hipStream_t st);
// words[0..n-1] = 0 by a small kernel (usable where a memset node is not: under graph capture)
hipError_t launch_clear_words(unsigned* words, int n, hipStream_t st);

}  // namespace pipesd
