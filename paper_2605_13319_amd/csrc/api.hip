// Host side of the NAV library: handles, paged-KV bookkeeping, the per-pass launch sequence.
#include <math.h>
#include <stdio.h>
#include <string.h>

#include <new>
#include <vector>

#include "common.h"

using namespace pipesd;

// text of the most recent failing HIP call of this thread, for pipesd_last_hip_error()
static thread_local char g_hip_msg[256] = "";
static int hip_fail(hipError_t e, const char* what) {
  snprintf(g_hip_msg, sizeof(g_hip_msg), "%s: %s", what, hipGetErrorString(e));
  return PIPESD_EHIP;
}

#define HIP_TRY(expr)                                 \
  do {                                                \
    hipError_t _e = (expr);                           \
    if (_e != hipSuccess) return hip_fail(_e, #expr); \
  } while (0)

extern "C" const char* pipesd_last_hip_error(void) { return g_hip_msg; }

// ---------------------------------------------------------------------------------------------
// handles
// ---------------------------------------------------------------------------------------------
constexpr int kMaxBatchResults = 256;  // decisions one batched call can return

struct pipesd_model {
  pipesd_config cfg{};
  bool on_device = false;
  size_t esz = 2;
  // library-owned device copies
  void* tok_emb = nullptr;
  float* final_norm = nullptr;
  void* lm_head = nullptr;
  std::vector<float*> attn_norm, ffn_norm;
  std::vector<void*> wqkv, wo, wgu, wdown;  // fp32: row-major stacks; bf16: matrix-core tiles
  double* theta = nullptr;
  // activation workspace (rows x width, fp32)
  float *xres = nullptr, *hbuf = nullptr, *qkv = nullptr, *qbuf = nullptr, *attn_out = nullptr, *gu = nullptr,
        *act2 = nullptr, *logits = nullptr, *rope_cs = nullptr;
  unsigned* counters = nullptr;
  ActArena arena{};  // bf16 path: per-layer activation buffers (passes of up to 32 rows)
  int pass_act_tiles = 2;  // row tiles of the buffers of the pass being enqueued
  ActArena arena_big{};  // bf16 path: one buffer of each kind, 16 row tiles (passes of several clients, up to 256 rows; 33..128 rows use 8 of them)
  int wide_mode = 0;        // GEMM kernel of passes of more than 64 rows: 0 by shape, 1 narrow, 2 wide
  void* wide_ws = nullptr;  // bf16 path: running sums of the K-split workgroups of passes of more than 64 rows
  size_t wide_ws_bytes = 0;
  RowMap* rowmap_dev = nullptr;  // bf16 path: per-row placement of a pass that holds several clients
  float* attn_part = nullptr;
  size_t attn_part_floats = 0;
  unsigned* attn_count = nullptr;  // arrival counters of the streaming attention kernel (zero between launches)
  // a pass begun by pipesd_nav_verify_begin and not yet ended (the model's buffers are in use by it)
  struct Pending {
    bool active = false;
    pipesd_kv* kv = nullptr;
    int32_t seq = 0, k = 0, text_len = 0;
    std::vector<int32_t> drafts;
    hipStream_t st = nullptr;
  } pending;
  int32_t* chain_alive = nullptr;  // bf16 path: one word per round of a chain (round r runs iff word r holds 1)
  const int32_t* gate = nullptr;   // the word the launches being enqueued are gated by (nullptr: they always run)
  float* row_stats = nullptr;
  unsigned long long* scan_partial = nullptr;
  int32_t* result_dev = nullptr;
  int32_t* result_host = nullptr;  // pinned
  std::vector<void*> owned;
  // fused layer kernel (bf16, passes of up to 16 rows)
  LayerSlabs slabs{};
  unsigned* bar = nullptr;
  unsigned long long* step_clock = nullptr;  // [4 * n_layers + 1] clocks of the last fused launch
  bool steps_recorded = false;
  bool fused_enabled = false;  // opt-in until it beats the per-projection launches
  int64_t fused_launches = 0, fused_checked = 0;
  // kernel timing
  int prof_class = PIPESD_PROF_OFF;
  std::vector<std::pair<hipEvent_t, hipEvent_t>> prof_events;
  size_t prof_used = 0;
};

struct SeqState {
  std::vector<int32_t> text;    // committed tokens; all but the last are cached, the last is pending
  std::vector<int32_t> blocks;  // KV blocks in position order
  int32_t table_synced = 0;     // block-table entries already mirrored on the device
};

struct pipesd_kv {
  const pipesd_model* model = nullptr;
  int32_t max_seqs = 0, n_blocks = 0;
  void* pool = nullptr;
  std::vector<int32_t> free_list;
  std::vector<SeqState> seqs;
  int32_t* table_dev = nullptr;  // [max_seqs][n_blocks]
  int64_t layer_stride = 0, v_offset = 0;
  int32_t block_elems = 0;
};

static constexpr int kCounterSlots = 1 << 16;

static int dev_alloc(pipesd_model* m, void** p, size_t bytes) {
  if (hipMalloc(p, bytes ? bytes : 256) != hipSuccess) return PIPESD_ENOMEM;
  m->owned.push_back(*p);
  return PIPESD_OK;
}

static int check_config(const pipesd_config* c) {
  if (c->n_layers < 1 || c->d_model < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1 || c->head_dim < 2 ||
      c->d_ffn < 1 || c->vocab < 1)
    return PIPESD_EINVAL;
  if (c->n_q_heads % c->n_kv_heads != 0 || (c->head_dim & 1) || c->head_dim > 128) return PIPESD_EINVAL;
  if (c->dtype != PIPESD_F32 && c->dtype != PIPESD_BF16) return PIPESD_EINVAL;
  if (!(c->rms_eps >= 0.f) || !(c->rope_base > 0.f)) return PIPESD_EINVAL;
  if (c->dtype == PIPESD_BF16) {
    const int qd = c->n_q_heads * c->head_dim;
    if (c->d_model % 512 || qd % 512 || c->d_ffn % 512) return PIPESD_EINVAL;
    if (c->head_dim != 64 && c->head_dim != 128) return PIPESD_EINVAL;
    if (c->d_model / 16 > 512) return PIPESD_EINVAL;  // the fused norm reads at most 512 partial sums of squares per row
  } else {
    if (c->d_model % 4 || c->d_ffn % 4) return PIPESD_EINVAL;
  }
  return PIPESD_OK;
}

static void model_free(pipesd_model* m) {
  if (!m) return;
  for (void* p : m->owned) (void)hipFree(p);
  if (m->attn_part) (void)hipFree(m->attn_part);  // (grown on demand, so not in `owned`)
  if (m->result_host) (void)hipHostFree(m->result_host);
  for (auto& e : m->prof_events) {
    (void)hipEventDestroy(e.first);
    (void)hipEventDestroy(e.second);
  }
  delete m;
}

static int copy_dev(pipesd_model* m, void** dst, const void* src, size_t bytes) {
  int rc = dev_alloc(m, dst, bytes);
  if (rc) return rc;
  HIP_TRY(hipMemcpy(*dst, src, bytes, hipMemcpyDeviceToDevice));
  return PIPESD_OK;
}

static int build_device_model(pipesd_model* m, const pipesd_weights* w) {
  const pipesd_config& c = m->cfg;
  const size_t e = m->esz;
  const int d = c.d_model, qd = c.n_q_heads * c.head_dim, kvd = c.n_kv_heads * c.head_dim, F = c.d_ffn, V = c.vocab;
  const int L = c.n_layers;
  if (!w->tok_emb || !w->final_norm || !w->lm_head || !w->attn_norm || !w->ffn_norm || !w->wq || !w->wk || !w->wv ||
      !w->wo || !w->w_gate || !w->w_up || !w->w_down)
    return PIPESD_EINVAL;
  for (int l = 0; l < L; ++l)
    if (!w->attn_norm[l] || !w->ffn_norm[l] || !w->wq[l] || !w->wk[l] || !w->wv[l] || !w->wo[l] || !w->w_gate[l] ||
        !w->w_up[l] || !w->w_down[l])
      return PIPESD_EINVAL;
  int rc;
  if ((rc = copy_dev(m, &m->tok_emb, w->tok_emb, (size_t)V * d * e))) return rc;
  if ((rc = copy_dev(m, (void**)&m->final_norm, w->final_norm, (size_t)d * 4))) return rc;
  m->attn_norm.resize(L);
  m->ffn_norm.resize(L);
  m->wqkv.resize(L);
  m->wo.resize(L);
  m->wgu.resize(L);
  m->wdown.resize(L);
  const int nqkv = qd + 2 * kvd;
  if (c.dtype == PIPESD_F32) {
    if ((rc = copy_dev(m, &m->lm_head, w->lm_head, (size_t)V * d * e))) return rc;
  } else {
    const int nt = (V + 15) / 16;
    if ((rc = dev_alloc(m, &m->lm_head, (size_t)nt * 16 * d * e))) return rc;
    PackSrc ps{{(const uint16_t*)w->lm_head, nullptr, nullptr}, {V, 0, 0}};
    HIP_TRY(launch_pack_bf16(ps, 1, d, PACK_PLAIN, 0, m->lm_head, nt, nullptr));
  }
  // bf16: one slab per kind of tensor, layer l at l * (bytes of one layer), so that device code
  // reaches a layer's weights by arithmetic instead of through a pointer table
  LayerSlabs& sl = m->slabs;
  if (c.dtype == PIPESD_BF16) {
    sl.qkv_bytes = (size_t)nqkv * d * e;
    sl.o_bytes = (size_t)d * qd * e;
    sl.gu_bytes = (size_t)2 * F * d * e;
    sl.down_bytes = (size_t)d * F * e;
    sl.norm_bytes = (size_t)d * 4;
    if ((rc = dev_alloc(m, (void**)&sl.wqkv, sl.qkv_bytes * L))) return rc;
    if ((rc = dev_alloc(m, (void**)&sl.wo, sl.o_bytes * L))) return rc;
    if ((rc = dev_alloc(m, (void**)&sl.wgu, sl.gu_bytes * L))) return rc;
    if ((rc = dev_alloc(m, (void**)&sl.wdown, sl.down_bytes * L))) return rc;
    if ((rc = dev_alloc(m, (void**)&sl.attn_norm, sl.norm_bytes * L))) return rc;
    if ((rc = dev_alloc(m, (void**)&sl.ffn_norm, sl.norm_bytes * L))) return rc;
  }
  for (int l = 0; l < L; ++l) {
    if (c.dtype == PIPESD_BF16) {
      m->attn_norm[l] = (float*)(sl.attn_norm + l * sl.norm_bytes);
      m->ffn_norm[l] = (float*)(sl.ffn_norm + l * sl.norm_bytes);
      HIP_TRY(hipMemcpy(m->attn_norm[l], w->attn_norm[l], sl.norm_bytes, hipMemcpyDeviceToDevice));
      HIP_TRY(hipMemcpy(m->ffn_norm[l], w->ffn_norm[l], sl.norm_bytes, hipMemcpyDeviceToDevice));
    } else {
      if ((rc = copy_dev(m, (void**)&m->attn_norm[l], w->attn_norm[l], (size_t)d * 4))) return rc;
      if ((rc = copy_dev(m, (void**)&m->ffn_norm[l], w->ffn_norm[l], (size_t)d * 4))) return rc;
    }
    if (c.dtype == PIPESD_F32) {
      if ((rc = dev_alloc(m, &m->wqkv[l], (size_t)nqkv * d * e))) return rc;
      char* p = (char*)m->wqkv[l];
      HIP_TRY(hipMemcpy(p, w->wq[l], (size_t)qd * d * e, hipMemcpyDeviceToDevice));
      HIP_TRY(hipMemcpy(p + (size_t)qd * d * e, w->wk[l], (size_t)kvd * d * e, hipMemcpyDeviceToDevice));
      HIP_TRY(hipMemcpy(p + (size_t)(qd + kvd) * d * e, w->wv[l], (size_t)kvd * d * e, hipMemcpyDeviceToDevice));
      if ((rc = copy_dev(m, &m->wo[l], w->wo[l], (size_t)d * qd * e))) return rc;
      if ((rc = dev_alloc(m, &m->wgu[l], (size_t)2 * F * d * e))) return rc;
      p = (char*)m->wgu[l];
      HIP_TRY(hipMemcpy(p, w->w_gate[l], (size_t)F * d * e, hipMemcpyDeviceToDevice));
      HIP_TRY(hipMemcpy(p + (size_t)F * d * e, w->w_up[l], (size_t)F * d * e, hipMemcpyDeviceToDevice));
      if ((rc = copy_dev(m, &m->wdown[l], w->w_down[l], (size_t)d * F * e))) return rc;
    } else {
      m->wqkv[l] = sl.wqkv + l * sl.qkv_bytes;
      m->wo[l] = sl.wo + l * sl.o_bytes;
      m->wgu[l] = sl.wgu + l * sl.gu_bytes;
      m->wdown[l] = sl.wdown + l * sl.down_bytes;
      PackSrc pq{{(const uint16_t*)w->wq[l], (const uint16_t*)w->wk[l], (const uint16_t*)w->wv[l]}, {qd, kvd, kvd}};
      HIP_TRY(launch_pack_bf16(pq, 3, d, PACK_HALVES, c.head_dim / 2, m->wqkv[l], nqkv / 16, nullptr));
      PackSrc po{{(const uint16_t*)w->wo[l], nullptr, nullptr}, {d, 0, 0}};
      HIP_TRY(launch_pack_bf16(po, 1, qd, PACK_PLAIN, 0, m->wo[l], d / 16, nullptr));
      PackSrc pg{{(const uint16_t*)w->w_gate[l], (const uint16_t*)w->w_up[l], nullptr}, {F, F, 0}};
      HIP_TRY(launch_pack_bf16(pg, 2, d, PACK_HALVES, F, m->wgu[l], 2 * F / 16, nullptr));
      PackSrc pd{{(const uint16_t*)w->w_down[l], nullptr, nullptr}, {d, 0, 0}};
      HIP_TRY(launch_pack_bf16(pd, 1, F, PACK_PLAIN, 0, m->wdown[l], d / 16, nullptr));
    }
  }
  // rotary frequencies theta_i = base^(-2i/h), fp64
  std::vector<double> th(c.head_dim / 2);
  for (int i = 0; i < c.head_dim / 2; ++i) th[i] = pow((double)c.rope_base, -2.0 * i / c.head_dim);
  if ((rc = dev_alloc(m, (void**)&m->theta, th.size() * 8))) return rc;
  HIP_TRY(hipMemcpy(m->theta, th.data(), th.size() * 8, hipMemcpyHostToDevice));

  const size_t R = kMaxRows;
  if ((rc = dev_alloc(m, (void**)&m->xres, R * d * 4))) return rc;
  if ((rc = dev_alloc(m, (void**)&m->hbuf, R * (size_t)(d > qd ? d : qd) * 4))) return rc;
  if ((rc = dev_alloc(m, (void**)&m->qkv, R * nqkv * 4))) return rc;
  if ((rc = dev_alloc(m, (void**)&m->qbuf, R * qd * 4))) return rc;
  if ((rc = dev_alloc(m, (void**)&m->attn_out, R * qd * 4))) return rc;
  if ((rc = dev_alloc(m, (void**)&m->gu, R * 2 * (size_t)F * 4))) return rc;
  if ((rc = dev_alloc(m, (void**)&m->act2, R * (size_t)F * 4))) return rc;
  const size_t RP = c.dtype == PIPESD_BF16 ? kMaxPassRows : kMaxRows;  // rows of the largest pass
  if ((rc = dev_alloc(m, (void**)&m->logits, RP * (size_t)V * 4))) return rc;
  if ((rc = dev_alloc(m, (void**)&m->rope_cs, RP * c.head_dim * 4))) return rc;
  // decision scratch: softmax partials of every row of the largest pass, scan sums per client
  if ((rc = dev_alloc(m, (void**)&m->row_stats, ((size_t)kMaxPassRows * 64 * 2 + 64) * 4))) return rc;
  if ((rc = dev_alloc(m, (void**)&m->scan_partial, (size_t)kMaxPassClients * 64 * 8))) return rc;
  if ((rc = dev_alloc(m, (void**)&m->result_dev, (size_t)2 * kMaxBatchResults * 4))) return rc;
  if ((rc = dev_alloc(m, (void**)&m->counters, (size_t)kCounterSlots * 4))) return rc;
  HIP_TRY(hipMemset(m->counters, 0, (size_t)kCounterSlots * 4));
  if (c.dtype == PIPESD_BF16) {
    if (device_cu_count() <= 0) return PIPESD_EHIP;
    const size_t arena_bytes = act_arena_layout(m->arena, L, d, qd, F, true, 2);
    if ((rc = dev_alloc(m, (void**)&m->arena.base, arena_bytes))) return rc;
    HIP_TRY(hipMemset(m->arena.base, 0, arena_bytes));
    const size_t big_bytes = act_arena_layout(m->arena_big, L, d, qd, F, false, kMaxPassRows / 16);
    if ((rc = dev_alloc(m, (void**)&m->arena_big.base, big_bytes))) return rc;
    HIP_TRY(hipMemset(m->arena_big.base, 0, big_bytes));
    const int gemm_nk[5][2] = {{(int)nqkv, (int)d}, {(int)d, (int)qd}, {2 * (int)F, (int)d}, {(int)d, (int)F}, {(int)V, (int)d}};
    for (const auto& nk : gemm_nk) m->wide_ws_bytes = std::max(m->wide_ws_bytes, gemm_wide_workspace_bytes(nk[0], nk[1]));  // (sized as if every product ran wide)
    if (m->wide_ws_bytes && (rc = dev_alloc(m, &m->wide_ws, m->wide_ws_bytes))) return rc;
    if ((rc = dev_alloc(m, (void**)&m->step_clock, ((size_t)4 * L + 1) * 8))) return rc;
    if ((rc = dev_alloc(m, (void**)&m->rowmap_dev, sizeof(RowMap)))) return rc;
    if ((rc = dev_alloc(m, (void**)&m->attn_count, kAttnCounters * sizeof(unsigned)))) return rc;
    HIP_TRY(hipMemset(m->attn_count, 0, kAttnCounters * sizeof(unsigned)));
    if ((rc = dev_alloc(m, (void**)&m->chain_alive, 64 * sizeof(int32_t)))) return rc;
    HIP_TRY(hipMemset(m->chain_alive, 0, 64 * sizeof(int32_t)));
    if ((rc = dev_alloc(m, (void**)&m->bar, 4096))) return rc;
    HIP_TRY(hipMemset(m->bar, 0, 4096));
  }
  HIP_TRY(hipHostMalloc((void**)&m->result_host, (size_t)(4 + 2 * kMaxBatchResults) * 4, hipHostMallocDefault));
  HIP_TRY(hipDeviceSynchronize());
  return PIPESD_OK;
}

extern "C" int pipesd_model_create(const pipesd_config* cfg, const pipesd_weights* weights, pipesd_model** out) {
  if (!cfg || !out) return PIPESD_EINVAL;
  int rc = check_config(cfg);
  if (rc) return rc;
  pipesd_model* m = new (std::nothrow) pipesd_model();
  if (!m) return PIPESD_ENOMEM;
  m->cfg = *cfg;
  m->esz = cfg->dtype == PIPESD_F32 ? 4 : 2;
  if (weights) {
    rc = build_device_model(m, weights);
    if (rc) {
      model_free(m);
      return rc;
    }
    m->on_device = true;
  }
  *out = m;
  return PIPESD_OK;
}

extern "C" int pipesd_model_destroy(pipesd_model* model) {
  if (!model) return PIPESD_EINVAL;
  if (model->on_device) (void)hipDeviceSynchronize();
  model_free(model);
  return PIPESD_OK;
}

extern "C" size_t pipesd_kv_block_bytes(const pipesd_model* model, int32_t block_tokens) {
  if (!model || block_tokens != kBlockTokens) return 0;
  const pipesd_config& c = model->cfg;
  return (size_t)c.n_layers * 2 * c.n_kv_heads * c.head_dim * block_tokens * model->esz;
}

static int ensure_attn_scratch(pipesd_model* m, size_t floats);

// Floats of attention partials the largest pass over a pool of `pool_tokens` cached tokens can need:
// a client brings at most kMaxRows rows and ceil(context / chunk) splits, the contexts of the
// clients of a pass add up to at most the pool, and a pass holds at most kMaxPassClients clients.
static size_t attn_scratch_bound(const pipesd_model* m, int64_t pool_tokens) {
  const int chunk = attn_chunk_tokens(m->cfg.dtype);
  const int64_t clients = m->cfg.dtype == PIPESD_BF16 ? kMaxPassClients : 1;
  const int64_t splits = pool_tokens / chunk + clients;
  // (the streaming kernel splits no finer but rounds a head group's rows up to whole pairs of 16-row tiles)
  const int64_t group_rows = (int64_t)(m->cfg.n_q_heads / m->cfg.n_kv_heads) * kMaxRows + 31;
  return (size_t)splits * (size_t)(group_rows * m->cfg.n_kv_heads) * (m->cfg.head_dim + 4);
}

extern "C" int pipesd_kv_create(const pipesd_model* model, int32_t max_seqs, int32_t block_tokens, void* pool,
                                size_t pool_bytes, pipesd_kv** out) {
  if (!model || !out || max_seqs < 1 || block_tokens != kBlockTokens) return PIPESD_EINVAL;
  const size_t bb = pipesd_kv_block_bytes(model, block_tokens);
  if (pool_bytes / bb < 1 || pool_bytes / bb > 0x7fffffff) return PIPESD_EINVAL;
  if (pool && ((uintptr_t)pool & 255)) return PIPESD_EINVAL;
  if (pool && !model->on_device) return PIPESD_ESTATE;
  pipesd_kv* kv = new (std::nothrow) pipesd_kv();
  if (!kv) return PIPESD_ENOMEM;
  kv->model = model;
  kv->max_seqs = max_seqs;
  kv->n_blocks = (int32_t)(pool_bytes / bb);
  kv->pool = pool;
  kv->seqs.resize(max_seqs);
  kv->free_list.reserve(kv->n_blocks);
  for (int32_t b = kv->n_blocks - 1; b >= 0; --b) kv->free_list.push_back(b);  // block 0 is handed out first
  const pipesd_config& c = model->cfg;
  kv->block_elems = c.n_kv_heads * kBlockTokens * c.head_dim;
  kv->v_offset = (int64_t)kv->n_blocks * kv->block_elems;
  kv->layer_stride = 2 * kv->v_offset;
  if (pool) {
    if (hipMalloc((void**)&kv->table_dev, (size_t)max_seqs * kv->n_blocks * 4) != hipSuccess) {
      delete kv;
      return PIPESD_ENOMEM;
    }
    if (hipMemset(kv->table_dev, 0, (size_t)max_seqs * kv->n_blocks * 4) != hipSuccess) {
      (void)hipFree(kv->table_dev);
      delete kv;
      return PIPESD_EHIP;
    }
    // the attention partials of any pass over this pool fit from now on: no verify call has to
    // synchronise the device and reallocate (the model handle is the library's own object)
    const int rc = ensure_attn_scratch(const_cast<pipesd_model*>(model), attn_scratch_bound(model, (int64_t)kv->n_blocks * kBlockTokens));
    if (rc) {
      (void)hipFree(kv->table_dev);
      delete kv;
      return rc;
    }
  }
  *out = kv;
  return PIPESD_OK;
}

extern "C" int pipesd_kv_destroy(pipesd_kv* kv) {
  if (!kv) return PIPESD_EINVAL;
  if (kv->table_dev) {
    (void)hipDeviceSynchronize();
    (void)hipFree(kv->table_dev);
  }
  delete kv;
  return PIPESD_OK;
}

static bool seq_ok(const pipesd_kv* kv, int32_t seq) { return kv && seq >= 0 && seq < kv->max_seqs; }

// blocks needed to hold `rows` cached rows
static int32_t blocks_for(int32_t rows) { return (rows + kBlockTokens - 1) / kBlockTokens; }

// give back every block wholly beyond `rows` cached rows
static void release_beyond(pipesd_kv* kv, SeqState& s, int32_t rows) {
  const int32_t keep = blocks_for(rows);
  while ((int32_t)s.blocks.size() > keep) {
    kv->free_list.push_back(s.blocks.back());
    s.blocks.pop_back();
  }
  if (s.table_synced > keep) s.table_synced = keep;
}

// a pass begun on this pool and not yet ended still writes the sequences' blocks
static bool pass_pending(const pipesd_kv* kv) { return kv->model && kv->model->pending.active && kv->model->pending.kv == kv; }

extern "C" int pipesd_seq_reset(pipesd_kv* kv, int32_t seq) {
  if (!seq_ok(kv, seq)) return PIPESD_EINVAL;
  if (pass_pending(kv)) return PIPESD_ESTATE;
  SeqState& s = kv->seqs[seq];
  release_beyond(kv, s, 0);
  s.text.clear();
  return PIPESD_OK;
}

extern "C" int pipesd_kv_rollback(pipesd_kv* kv, int32_t seq, int32_t new_prefix_len) {
  if (!seq_ok(kv, seq)) return PIPESD_EINVAL;
  if (pass_pending(kv)) return PIPESD_ESTATE;
  SeqState& s = kv->seqs[seq];
  if (new_prefix_len < 1 || new_prefix_len > (int32_t)s.text.size()) return PIPESD_ESTATE;
  s.text.resize(new_prefix_len);
  release_beyond(kv, s, new_prefix_len - 1);
  return PIPESD_OK;
}

extern "C" int pipesd_kv_len(const pipesd_kv* kv, int32_t seq, int32_t* prefix_len) {
  if (!seq_ok(kv, seq) || !prefix_len) return PIPESD_EINVAL;
  *prefix_len = (int32_t)kv->seqs[seq].text.size();
  return PIPESD_OK;
}

extern "C" int pipesd_kv_free_blocks(const pipesd_kv* kv, int32_t* n_free) {
  if (!kv || !n_free) return PIPESD_EINVAL;
  *n_free = (int32_t)kv->free_list.size();
  return PIPESD_OK;
}

extern "C" int pipesd_kv_seq_blocks(const pipesd_kv* kv, int32_t seq, int32_t* n_blocks) {
  if (!seq_ok(kv, seq) || !n_blocks) return PIPESD_EINVAL;
  *n_blocks = (int32_t)kv->seqs[seq].blocks.size();
  return PIPESD_OK;
}

extern "C" const char* pipesd_strerror(int status) {
  switch (status) {
    case PIPESD_OK: return "ok";
    case PIPESD_EINVAL: return "invalid argument";
    case PIPESD_ENOMEM: return "out of KV blocks or device memory";
    case PIPESD_ESTATE: return "call does not fit the sequence state";
    case PIPESD_EHIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

// ---------------------------------------------------------------------------------------------
// kernel timing
// ---------------------------------------------------------------------------------------------
extern "C" int pipesd_model_set_wide_gemm(pipesd_model* model, int32_t mode) {
  if (!model || mode < 0 || mode > 2) return PIPESD_EINVAL;
  model->wide_mode = mode;
  return PIPESD_OK;
}

extern "C" int pipesd_model_set_fused(pipesd_model* model, int32_t on) {
  if (!model) return PIPESD_EINVAL;
  model->fused_enabled = on != 0;
  return PIPESD_OK;
}

extern "C" int pipesd_model_fused_launches(const pipesd_model* model, int64_t* n) {
  if (!model || !n) return PIPESD_EINVAL;
  *n = model->fused_launches;
  return PIPESD_OK;
}

extern "C" int pipesd_profile_select(pipesd_model* model, int32_t kernel_class) {
  if (!model || kernel_class < PIPESD_PROF_OFF || kernel_class > PIPESD_PROF_LAYERS) return PIPESD_EINVAL;
  model->prof_class = kernel_class;
  model->prof_used = 0;
  return PIPESD_OK;
}

extern "C" int pipesd_profile_read(pipesd_model* model, int32_t* n_launches, double* total_ms) {
  if (!model || !n_launches || !total_ms) return PIPESD_EINVAL;
  double tot = 0.0;
  for (size_t i = 0; i < model->prof_used; ++i) {
    HIP_TRY(hipEventSynchronize(model->prof_events[i].second));
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, model->prof_events[i].first, model->prof_events[i].second));
    tot += ms;
  }
  *n_launches = (int32_t)model->prof_used;
  *total_ms = tot;
  model->prof_used = 0;
  return PIPESD_OK;
}

extern "C" int pipesd_profile_read_each(pipesd_model* model, double* us_out, int32_t cap, int32_t* n_launches) {
  if (!model || !n_launches || cap < 0 || (cap > 0 && !us_out)) return PIPESD_EINVAL;
  for (size_t i = 0; i < model->prof_used; ++i) {
    HIP_TRY(hipEventSynchronize(model->prof_events[i].second));
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, model->prof_events[i].first, model->prof_events[i].second));
    if ((int64_t)i < cap) us_out[i] = (double)ms * 1e3;
  }
  *n_launches = (int32_t)model->prof_used;
  model->prof_used = 0;
  return PIPESD_OK;
}

extern "C" int pipesd_profile_read_steps(pipesd_model* model, double* us_out, int32_t cap, int32_t* n_steps) {
  if (!model || !us_out || !n_steps || cap < 0) return PIPESD_EINVAL;
  *n_steps = 0;
  if (!model->step_clock || !model->steps_recorded) return PIPESD_OK;
  const int n = 4 * model->cfg.n_layers;
  std::vector<unsigned long long> clk((size_t)n + 1);
  HIP_TRY(hipDeviceSynchronize());
  HIP_TRY(hipMemcpy(clk.data(), model->step_clock, clk.size() * 8, hipMemcpyDeviceToHost));
  int dev = 0, khz = 0;
  HIP_TRY(hipGetDevice(&dev));
  HIP_TRY(hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev));
  if (khz <= 0) return PIPESD_EHIP;
  for (int i = 0; i < n && i < cap; ++i) us_out[i] = (double)(clk[i + 1] - clk[i]) * 1e3 / (double)khz;
  *n_steps = n;
  return PIPESD_OK;
}

namespace {
struct ProfScope {
  pipesd_model* m;
  hipStream_t st;
  bool on;
  ProfScope(pipesd_model* m_, int cls, hipStream_t st_) : m(m_), st(st_) {
    on = m->prof_class != PIPESD_PROF_OFF &&
         (m->prof_class == cls || (m->prof_class == PIPESD_PROF_ALL_GEMM && cls >= PIPESD_PROF_GEMM_QKV &&
                                   cls <= PIPESD_PROF_GEMM_LMHEAD));
    if (!on) return;
    if (m->prof_used == m->prof_events.size()) {
      hipEvent_t a, b;
      if (hipEventCreate(&a) != hipSuccess) {
        on = false;
        return;
      }
      if (hipEventCreate(&b) != hipSuccess) {
        (void)hipEventDestroy(a);
        on = false;
        return;
      }
      m->prof_events.emplace_back(a, b);
    }
    (void)hipEventRecord(m->prof_events[m->prof_used].first, st);
  }
  ~ProfScope() {
    if (!on) return;
    (void)hipEventRecord(m->prof_events[m->prof_used].second, st);
    ++m->prof_used;
  }
};
// a GEMM launch of the selected class carries its own start / stop events instead
struct ProfGemm {
  pipesd_model* m;
  bool on;
  ProfGemm(pipesd_model* m_, int cls, GemmCall& g) : m(m_) {
    on = m->prof_class != PIPESD_PROF_OFF &&
         (m->prof_class == cls || (m->prof_class == PIPESD_PROF_ALL_GEMM && cls >= PIPESD_PROF_GEMM_QKV &&
                                   cls <= PIPESD_PROF_GEMM_LMHEAD));
    if (!on) return;
    if (m->prof_used == m->prof_events.size()) {
      hipEvent_t a, b;
      if (hipEventCreate(&a) != hipSuccess) {
        on = false;
        return;
      }
      if (hipEventCreate(&b) != hipSuccess) {
        (void)hipEventDestroy(a);
        on = false;
        return;
      }
      m->prof_events.emplace_back(a, b);
    }
    g.ev_start = m->prof_events[m->prof_used].first;
    g.ev_stop = m->prof_events[m->prof_used].second;
  }
  ~ProfGemm() {
    if (on) ++m->prof_used;
  }
};
}  // namespace

// ---------------------------------------------------------------------------------------------
// the forward over a row block
// ---------------------------------------------------------------------------------------------
static KvView view_of(const pipesd_kv* kv, int32_t seq) {
  KvView v;
  v.pool = kv->pool;
  v.table = kv->table_dev + (size_t)seq * kv->n_blocks;
  v.layer_stride = kv->layer_stride;
  v.v_offset = kv->v_offset;
  v.block_elems = kv->block_elems;
  v.n_kv_heads = kv->model->cfg.n_kv_heads;
  v.head_dim = kv->model->cfg.head_dim;
  return v;
}

// make sure the sequence owns blocks for `rows` cached rows and the device table shows them
static int ensure_blocks(pipesd_kv* kv, int32_t seq, int32_t rows, hipStream_t st) {
  SeqState& s = kv->seqs[seq];
  const int32_t need = blocks_for(rows);
  const int32_t have = (int32_t)s.blocks.size();
  if (need - have > (int32_t)kv->free_list.size()) return PIPESD_ENOMEM;
  for (int32_t i = have; i < need; ++i) {
    s.blocks.push_back(kv->free_list.back());
    kv->free_list.pop_back();
  }
  if (kv->table_dev && s.table_synced < (int32_t)s.blocks.size()) {
    const int32_t first = s.table_synced, n = (int32_t)s.blocks.size() - first;
    HIP_TRY(launch_set_table(kv->table_dev + (size_t)seq * kv->n_blocks, first, s.blocks.data() + first, n, st));
    s.table_synced = (int32_t)s.blocks.size();
  }
  return PIPESD_OK;
}

static int ensure_attn_scratch(pipesd_model* m, size_t floats) {
  if (floats <= m->attn_part_floats) return PIPESD_OK;
  HIP_TRY(hipDeviceSynchronize());
  if (m->attn_part) (void)hipFree(m->attn_part);
  m->attn_part = nullptr;
  m->attn_part_floats = 0;
  const size_t want = floats + floats / 2;
  if (hipMalloc((void**)&m->attn_part, want * 4) != hipSuccess) return PIPESD_ENOMEM;
  m->attn_part_floats = want;
  return PIPESD_OK;
}

static GemmCall gemm_call(pipesd_model* m, const void* wp, int N, int K, int rows, const void* actp,
                          const float* ssq_in, int norm_parts, int epi) {
  GemmCall c{};
  c.wp = wp;
  c.N = N;
  c.K = K;
  c.m = rows;
  c.actp = actp;
  c.act_tiles = m->pass_act_tiles;
  c.ssq_in = ssq_in;
  c.ssq_parts = norm_parts;
  c.ssq_stride = m->arena.ssq_stride;
  c.eps = m->cfg.rms_eps;
  c.epi = epi;
  c.rope_cs = m->rope_cs;
  c.wide_ws = m->wide_ws;
  c.wide_ws_bytes = m->wide_ws_bytes;
  c.wide_mode = m->wide_mode;
  c.gate = m->gate;
  return c;
}

// The rows of one pass: one client's k + 1 rows, or (bf16) the rows of up to 16 clients one after
// the other, at most 128 in all.
constexpr int kPrefillRows = 128;  // rows per pass of prompt ingestion (bf16)
struct PassClient {
  int32_t seq, rows, start_pos;
};
struct PassLayout {
  int n_clients = 0, rows = 0;
  PassClient client[kMaxPassClients];
  PassTokens tok{};
};
constexpr int kPassRowsCap = 256;  // rows the batched call puts into one pass (<= kMaxPassRows)

static int run_pass(pipesd_model* m, pipesd_kv* kv, const PassLayout& pl, bool want_logits, hipStream_t st) {
  const pipesd_config& c = m->cfg;
  const int d = c.d_model, qd = c.n_q_heads * c.head_dim, kvd = c.n_kv_heads * c.head_dim, F = c.d_ffn, V = c.vocab;
  const int nqkv = qd + 2 * kvd;
  const int rows = pl.rows;
  const bool bf = c.dtype == PIPESD_BF16;
  const bool single = pl.n_clients == 1;
  if (pl.n_clients < 1 || pl.n_clients > kMaxPassClients || rows < 1 || rows > (bf ? kMaxPassRows : kMaxRows) ||
      (!bf && !single))
    return PIPESD_EINVAL;
  const int32_t seq = pl.client[0].seq;
  const int start_pos = pl.client[0].start_pos;
  // one client: the block table pointer is the client's own; several: the tables' common base + an offset per row
  KvView view = view_of(kv, single ? seq : 0);
  const int chunk = attn_chunk_tokens(c.dtype);
  const int nsplit = attn_nsplit(start_pos + rows, chunk);  // (one client)
  RowMap map{};
  AttnBatch ab{};
  ab.n = pl.n_clients;
  size_t part_floats = 0;
  for (int i = 0, r0 = 0; i < pl.n_clients; ++i) {
    const PassClient& pc = pl.client[i];
    const int32_t toff = single ? 0 : pc.seq * kv->n_blocks;
    for (int r = 0; r < pc.rows; ++r) {
      map.pos[r0 + r] = pc.start_pos + r;
      map.table_off[r0 + r] = toff;
    }
    AttnClient& ac = ab.c[i];
    ac.row_off = r0;
    ac.m = pc.rows;
    ac.start_pos = pc.start_pos;
    ac.table_off = toff;
    ac.nsplit = attn_nsplit(pc.start_pos + pc.rows, chunk);
    if (part_floats > (size_t)INT32_MAX) return PIPESD_ENOMEM;
    ac.part_off = (int32_t)part_floats;
    part_floats += (size_t)c.n_q_heads * pc.rows * ac.nsplit * (c.head_dim + 4);
    r0 += pc.rows;
  }
  // per-layer partial buffers only where the all-layers kernel may run (one client); otherwise one, reused
  const bool part_per_layer = bf && single && rows <= 16;
  // passes of few rows per client: the streaming attention kernel with its own split of every context
  AttnBatch ab_stream = ab;
  size_t stream_floats = 0;
  const bool may_fuse = bf && single && m->fused_enabled && m->gate == nullptr;
  const int stream_tiles = bf && !may_fuse ? attn_stream_plan(c.n_q_heads, c.n_kv_heads, c.head_dim, ab_stream, &stream_floats) : 0;
  int rc = ensure_attn_scratch(m, std::max(part_floats * (part_per_layer ? c.n_layers : 1), stream_tiles ? stream_floats : 0));
  if (rc) return rc;
  ActArena& ar = rows <= 2 * 16 ? m->arena : m->arena_big;
  const int act_tiles = rows <= 2 * 16 ? 2 : rows <= 8 * 16 ? 8 : kMaxPassRows / 16;
  m->pass_act_tiles = act_tiles;
  ar.part = m->attn_part;
  ar.part_stride = part_per_layer ? part_floats : 0;
  const RowMap* rows_dev = single ? nullptr : m->rowmap_dev;
  HIP_TRY(launch_setup_rows(c.dtype, m->tok_emb, pl.tok, map, rows, d, c.head_dim, m->theta, bf ? ar.ra(0) : m->xres,
                            m->rope_cs, bf ? m->attn_norm[0] : nullptr, bf ? ar.xa(0) : nullptr, act_tiles,
                            bf ? ar.sa(0) : nullptr, ar.ssq_stride, single ? nullptr : m->rowmap_dev, st));
  int norm_parts = 1;  // the row setup leaves one sum of squares per row, residual epilogues one per n-tile
  bool fused = false;
  if (bf && single && m->fused_enabled && m->gate == nullptr) {
    LayersCall lc{};
    lc.slabs = m->slabs;
    lc.final_norm = m->final_norm;
    lc.n_layers = c.n_layers;
    lc.m = rows;
    lc.start_pos = start_pos;
    lc.n_q_heads = c.n_q_heads;
    lc.head_dim = c.head_dim;
    lc.d_model = d;
    lc.q_dim = qd;
    lc.d_ffn = F;
    lc.eps = c.rms_eps;
    lc.kv = view;
    lc.rope_cs = m->rope_cs;
    lc.arena = ar;
    lc.bar = m->bar;
    lc.step_clock = m->prof_class == PIPESD_PROF_LAYERS ? m->step_clock : nullptr;
    if (layers_fused_supported(lc)) {
      ProfScope ps(m, PIPESD_PROF_LAYERS, st);
      HIP_TRY(launch_layers(lc, st));
      if (lc.step_clock) m->steps_recorded = true;
      ++m->fused_launches;
      fused = true;
      norm_parts = d / 16;
    }
  }
  for (int l = 0; l < (fused ? 0 : c.n_layers); ++l) {
    AttnCall at{};
    at.dtype = c.dtype;
    at.q = bf ? ar.q(l) : m->qbuf;
    at.kv = view;
    at.layer = l;
    at.m = rows;
    at.start_pos = start_pos;
    at.n_q_heads = c.n_q_heads;
    at.chunk = chunk;
    at.part = ar.partials(l);
    at.out = m->attn_out;
    at.outp = bf ? ar.ap(l) : nullptr;
    at.act_tiles = act_tiles;
    at.batch = stream_tiles ? ab_stream : ab;
    at.gate = m->gate;
    at.stream_tiles = stream_tiles;
    at.counters = m->attn_count;
    if (stream_tiles) at.part = m->attn_part;
    if (c.dtype == PIPESD_F32) {
      {
        ProfScope ps(m, PIPESD_PROF_GEMM_QKV, st);
        HIP_TRY(launch_rmsnorm_rows(m->xres, m->attn_norm[l], c.rms_eps, rows, d, m->hbuf, st));
        HIP_TRY(launch_gemm_f32(m->hbuf, d, (const float*)m->wqkv[l], nqkv, d, rows, m->qkv, nqkv, 0, st));
        HIP_TRY(launch_rope_append_f32(m->qkv, rows, start_pos, l, c.n_q_heads, view, m->rope_cs, m->qbuf, st));
      }
      {
        ProfScope ps(m, PIPESD_PROF_ATTN, st);
        HIP_TRY(launch_attention(at, st));
      }
      {
        ProfScope ps(m, PIPESD_PROF_GEMM_O, st);
        HIP_TRY(launch_gemm_f32(m->attn_out, qd, (const float*)m->wo[l], d, qd, rows, m->xres, d, 1, st));
      }
      {
        ProfScope ps(m, PIPESD_PROF_GEMM_GATEUP, st);
        HIP_TRY(launch_rmsnorm_rows(m->xres, m->ffn_norm[l], c.rms_eps, rows, d, m->hbuf, st));
        HIP_TRY(launch_gemm_f32(m->hbuf, d, (const float*)m->wgu[l], 2 * F, d, rows, m->gu, 2 * F, 0, st));
        HIP_TRY(launch_silu_mul(m->gu, rows, F, m->act2, st));
      }
      {
        ProfScope ps(m, PIPESD_PROF_GEMM_DOWN, st);
        HIP_TRY(launch_gemm_f32(m->act2, F, (const float*)m->wdown[l], d, F, rows, m->xres, d, 1, st));
      }
    } else {
      {
        GemmCall g = gemm_call(m, m->wqkv[l], nqkv, d, rows, ar.xa(l), ar.sa(l), norm_parts, EPI_QKV);
        ProfGemm pg(m, PIPESD_PROF_GEMM_QKV, g);
        g.out = ar.q(l);
        g.ldo = qd;
        g.rows = rows_dev;
        g.kv = view;
        g.layer = l;
        g.start_pos = start_pos;
        g.n_q_heads = c.n_q_heads;
        HIP_TRY(launch_gemm_bf16(g, st));
      }
      {
        ProfScope ps(m, PIPESD_PROF_ATTN, st);
        HIP_TRY(launch_attention(at, st));
      }
      {
        GemmCall g = gemm_call(m, m->wo[l], d, qd, rows, ar.ap(l), nullptr, 0, EPI_RESID);
        ProfGemm pg(m, PIPESD_PROF_GEMM_O, g);
        g.res_in = ar.ra(l);
        g.out = ar.rb(l);
        g.ldo = d;
        g.outp = ar.xb(l);
        g.gain_next = m->ffn_norm[l];
        g.ssq_out = ar.sb(l);
        HIP_TRY(launch_gemm_bf16(g, st));
        norm_parts = d / 16;
      }
      {
        GemmCall g = gemm_call(m, m->wgu[l], 2 * F, d, rows, ar.xb(l), ar.sb(l), norm_parts, EPI_SWIGLU);
        ProfGemm pg(m, PIPESD_PROF_GEMM_GATEUP, g);
        g.outp = ar.gp(l);
        HIP_TRY(launch_gemm_bf16(g, st));
      }
      {
        GemmCall g = gemm_call(m, m->wdown[l], d, F, rows, ar.gp(l), nullptr, 0, EPI_RESID);
        ProfGemm pg(m, PIPESD_PROF_GEMM_DOWN, g);
        g.res_in = ar.rb(l);
        g.out = ar.ra(l + 1);
        g.ldo = d;
        g.outp = ar.xa(l + 1);
        g.gain_next = l + 1 < c.n_layers ? m->attn_norm[l + 1] : m->final_norm;
        g.ssq_out = ar.sa(l + 1);
        HIP_TRY(launch_gemm_bf16(g, st));
      }
    }
  }
  if (want_logits) {
    if (c.dtype == PIPESD_F32) {
      ProfScope ps(m, PIPESD_PROF_GEMM_LMHEAD, st);
      HIP_TRY(launch_rmsnorm_rows(m->xres, m->final_norm, c.rms_eps, rows, d, m->hbuf, st));
      HIP_TRY(launch_gemm_f32(m->hbuf, d, (const float*)m->lm_head, V, d, rows, m->logits, V, 0, st));
    } else {
      GemmCall g = gemm_call(m, m->lm_head, V, d, rows, ar.xa(c.n_layers), ar.sa(c.n_layers), norm_parts, EPI_STORE);
      ProfGemm pg(m, PIPESD_PROF_GEMM_LMHEAD, g);
      g.out = m->logits;
      g.ldo = V;
      HIP_TRY(launch_gemm_bf16(g, st));
    }
  }
  return PIPESD_OK;
}

static int run_rows(pipesd_model* m, pipesd_kv* kv, int32_t seq, const int32_t* row_tokens, int rows, int start_pos,
                    bool want_logits, hipStream_t st) {
  PassLayout pl;
  pl.n_clients = 1;
  pl.rows = rows;
  pl.client[0] = PassClient{seq, rows, start_pos};
  for (int r = 0; r < rows; ++r) pl.tok.tok[r] = row_tokens[r];
  return run_pass(m, kv, pl, want_logits, st);
}

// The fused layer kernel raises a sticky flag if one of its device-wide barriers timed out.
static hipError_t read_layers_flag(pipesd_model* m, hipStream_t st) {
  m->result_host[2] = 0;
  if (!m->bar || m->fused_launches == m->fused_checked) return hipSuccess;
  m->fused_checked = m->fused_launches;
  return hipMemcpyAsync(m->result_host + 2, m->bar + kLayersErrWord, 4, hipMemcpyDeviceToHost, st);
}
static bool layers_flag_raised(pipesd_model* m) {
  if (m->result_host[2] == 0) return false;
  (void)hipMemset(m->bar + kLayersErrWord, 0, 4);
  return true;
}

static bool compute_ready(const pipesd_model* m, const pipesd_kv* kv) {
  return m && kv && kv->model == m && m->on_device && kv->pool && kv->table_dev && !m->pending.active;
}

extern "C" int pipesd_prefill(pipesd_model* model, pipesd_kv* kv, int32_t seq, const int32_t* tokens, int32_t n,
                              void* stream) {
  if (!model || !kv || !tokens || n < 1 || !seq_ok(kv, seq) || kv->model != model) return PIPESD_EINVAL;
  for (int32_t i = 0; i < n; ++i)
    if (tokens[i] < 0 || tokens[i] >= model->cfg.vocab) return PIPESD_EINVAL;
  if (!compute_ready(model, kv)) return PIPESD_ESTATE;
  hipStream_t st = (hipStream_t)stream;
  SeqState& s = kv->seqs[seq];
  const int32_t lp = (int32_t)s.text.size();
  std::vector<int32_t> rows;
  if (lp > 0) rows.push_back(s.text.back());
  rows.insert(rows.end(), tokens, tokens + n - 1);
  const int32_t start = lp > 0 ? lp - 1 : 0;
  const int32_t cached_before = start;
  int rc = ensure_blocks(kv, seq, start + (int32_t)rows.size(), st);
  if (rc) return rc;
  const size_t block = model->cfg.dtype == PIPESD_BF16 ? kPrefillRows : kMaxRows;  // rows per pass
  for (size_t i = 0; i < rows.size(); i += block) {
    const int nr = (int)((rows.size() - i < block) ? rows.size() - i : block);
    rc = run_rows(model, kv, seq, rows.data() + i, nr, start + (int)i, false, st);
    if (rc) {
      release_beyond(kv, s, cached_before);
      return rc;
    }
  }
  s.text.insert(s.text.end(), tokens, tokens + n);
  return PIPESD_OK;
}

static int verify_common(pipesd_model* model, pipesd_kv* kv, int32_t seq, const int32_t* extra, int32_t k,
                         int32_t* start_out, hipStream_t st) {
  SeqState& s = kv->seqs[seq];
  const int32_t lp = (int32_t)s.text.size();
  int32_t rows[kMaxRows];
  rows[0] = s.text.back();
  for (int32_t i = 0; i < k; ++i) rows[i + 1] = extra[i];
  int rc = ensure_blocks(kv, seq, lp + k, st);
  if (rc) return rc;
  rc = run_rows(model, kv, seq, rows, k + 1, lp - 1, true, st);
  if (rc) release_beyond(kv, s, lp - 1);
  *start_out = lp - 1;
  return rc;
}

constexpr int kMaxBatch = kMaxBatchResults;  // sequences per batched call

// host-side checks of one sequence's verify arguments (argument errors, then, if `state`, the
// handles' and the sequence's state); changes nothing
static int check_verify_args(const pipesd_model* model, const pipesd_kv* kv, int32_t seq, int32_t prefix_len,
                             const int32_t* draft_tokens, int32_t k, const float* draft_probs, const float* uniforms,
                             bool state = true) {
  if (!draft_tokens || !seq_ok(kv, seq)) return PIPESD_EINVAL;
  if (k < 1 || k > kMaxRows - 1) return PIPESD_EINVAL;
  if (draft_probs && !uniforms) return PIPESD_EINVAL;
  for (int32_t i = 0; i < k; ++i)
    if (draft_tokens[i] < 0 || draft_tokens[i] >= model->cfg.vocab) return PIPESD_EINVAL;
  if (draft_probs)
    for (int32_t i = 0; i <= k; ++i)
      if (!(uniforms[i] >= 0.f && uniforms[i] < 1.f)) return PIPESD_EINVAL;
  if (!state) return PIPESD_OK;
  if (!compute_ready(model, kv)) return PIPESD_ESTATE;
  const int32_t lp = (int32_t)kv->seqs[seq].text.size();
  if (lp < 1 || prefix_len != lp) return PIPESD_ESTATE;
  return PIPESD_OK;
}

// decision + cache trim of one sequence on logits rows [row_off, row_off + k] of the model's logits
// buffer, enqueued on `st`; the decision lands in result[0..1] on the device (and in result_copy)
static hipError_t enqueue_decision(pipesd_model* model, pipesd_kv* kv, int32_t seq, int32_t row_off, int32_t start,
                                   const int32_t* draft_tokens, int32_t k, const float* draft_probs,
                                   const float* uniforms, int32_t* result, int32_t* result_copy, hipStream_t st) {
  VerifyCall vc{};
  vc.logits_or_p = model->logits + (size_t)row_off * model->cfg.vocab;
  vc.q = draft_probs;
  vc.k = k;
  vc.V = model->cfg.vocab;
  for (int32_t i = 0; i < k; ++i) vc.drafts.tok[i] = draft_tokens[i];
  if (draft_probs)
    for (int32_t i = 0; i <= k; ++i) vc.u[i] = uniforms[i];
  vc.row_stats = model->row_stats;
  vc.scan_partial = model->scan_partial;
  vc.counter = model->counters + (kCounterSlots - 1);
  vc.result = result;
  vc.result_copy = result_copy;
  hipError_t e = hipSuccess;
  ProfScope ps(model, PIPESD_PROF_VERIFY, st);
  if (draft_probs) {
    vc.from_logits = true;  // probabilities are formed inside the decision kernel, never written out
    e = launch_softmax_stats(vc, st);
    if (e == hipSuccess) e = launch_spec_accept(vc, st);
  } else {
    e = launch_greedy_accept(vc, st);
  }
  if (e == hipSuccess)
    e = launch_kv_trim(model->cfg.dtype, view_of(kv, seq), model->cfg.n_layers, start, k, result, st);
  return e;
}

// forward + decision + cache trim of one sequence, enqueued on `st`.  On failure the sequence's
// block list is back to what it was.
static int enqueue_verify(pipesd_model* model, pipesd_kv* kv, int32_t seq, const int32_t* draft_tokens, int32_t k,
                          const float* draft_probs, const float* uniforms, int32_t* result, int32_t* result_copy,
                          hipStream_t st) {
  SeqState& s = kv->seqs[seq];
  const int32_t lp = (int32_t)s.text.size();
  int32_t start = 0;
  int rc = verify_common(model, kv, seq, draft_tokens, k, &start, st);
  if (rc) return rc;
  hipError_t e = enqueue_decision(model, kv, seq, 0, start, draft_tokens, k, draft_probs, uniforms, result, result_copy, st);
  if (e != hipSuccess) {
    release_beyond(kv, s, lp - 1);
    return hip_fail(e, "verify step");
  }
  return PIPESD_OK;
}

// after the stream has been synchronised: book the decision of one sequence
static int commit_verify(pipesd_model* model, pipesd_kv* kv, int32_t seq, const int32_t* draft_tokens, int32_t k,
                         const int32_t* result_host, int32_t* accepted_len, int32_t* next_token) {
  SeqState& s = kv->seqs[seq];
  const int32_t a = result_host[0], nxt = result_host[1];
  if (a < 0 || a > k || nxt < 0 || nxt >= model->cfg.vocab) return PIPESD_EHIP;
  const int32_t lp = (int32_t)s.text.size();
  s.text.insert(s.text.end(), draft_tokens, draft_tokens + a);
  s.text.push_back(nxt);
  release_beyond(kv, s, lp + a);
  *accepted_len = a;
  *next_token = nxt;
  return PIPESD_OK;
}

extern "C" int pipesd_nav_verify(pipesd_model* model, pipesd_kv* kv, int32_t seq, int32_t prefix_len,
                                 const int32_t* draft_tokens, int32_t k, const float* draft_probs,
                                 const float* uniforms, int32_t* accepted_len, int32_t* next_token, void* stream) {
  if (!model || !kv || !accepted_len || !next_token || kv->model != model) return PIPESD_EINVAL;
  int rc = check_verify_args(model, kv, seq, prefix_len, draft_tokens, k, draft_probs, uniforms);
  if (rc) return rc;
  SeqState& s = kv->seqs[seq];
  const int32_t lp = (int32_t)s.text.size();
  hipStream_t st = (hipStream_t)stream;
  model->result_host[0] = model->result_host[1] = -1;
  rc = enqueue_verify(model, kv, seq, draft_tokens, k, draft_probs, uniforms, model->result_dev, model->result_host, st);
  if (rc) return rc;
  hipError_t e = read_layers_flag(model, st);  // the decision itself lands in pinned host memory, written by the kernel
  if (e == hipSuccess) e = hipStreamSynchronize(st);
  if (e != hipSuccess) {
    release_beyond(kv, s, lp - 1);
    return hip_fail(e, "verify step");
  }
  if (layers_flag_raised(model)) {
    release_beyond(kv, s, lp - 1);
    return hip_fail(hipErrorLaunchFailure, "device-wide barrier of the fused layer kernel timed out");
  }
  rc = commit_verify(model, kv, seq, draft_tokens, k, model->result_host, accepted_len, next_token);
  if (rc) release_beyond(kv, s, lp - 1);
  return rc;
}

// The same pass in two halves: everything up to the last launch, and the wait + bookkeeping.
extern "C" int pipesd_nav_verify_begin(pipesd_model* model, pipesd_kv* kv, int32_t seq, int32_t prefix_len,
                                       const int32_t* draft_tokens, int32_t k, const float* draft_probs,
                                       const float* uniforms, void* stream) {
  if (!model || !kv || kv->model != model) return PIPESD_EINVAL;
  int rc = check_verify_args(model, kv, seq, prefix_len, draft_tokens, k, draft_probs, uniforms);
  if (rc) return rc;  // (ESTATE also while another pass is pending: compute_ready)
  SeqState& s = kv->seqs[seq];
  hipStream_t st = (hipStream_t)stream;
  model->result_host[0] = model->result_host[1] = -1;
  rc = enqueue_verify(model, kv, seq, draft_tokens, k, draft_probs, uniforms, model->result_dev, model->result_host, st);
  if (rc) return rc;
  const hipError_t e = read_layers_flag(model, st);
  if (e != hipSuccess) {
    (void)hipStreamSynchronize(st);
    release_beyond(kv, s, (int32_t)s.text.size() - 1);
    return hip_fail(e, "verify step");
  }
  model->pending.active = true;
  model->pending.kv = kv;
  model->pending.seq = seq;
  model->pending.k = k;
  model->pending.text_len = (int32_t)s.text.size();
  model->pending.drafts.assign(draft_tokens, draft_tokens + k);
  model->pending.st = st;
  return PIPESD_OK;
}

extern "C" int pipesd_nav_verify_done(pipesd_model* model, int32_t* done) {
  if (!model || !done) return PIPESD_EINVAL;
  if (!model->pending.active) return PIPESD_ESTATE;
  const hipError_t e = hipStreamQuery(model->pending.st);
  if (e != hipSuccess && e != hipErrorNotReady) return hip_fail(e, "verify step");
  *done = e == hipSuccess ? 1 : 0;
  return PIPESD_OK;
}

extern "C" int pipesd_nav_verify_end(pipesd_model* model, int32_t* accepted_len, int32_t* next_token) {
  if (!model || !accepted_len || !next_token) return PIPESD_EINVAL;
  if (!model->pending.active) return PIPESD_ESTATE;
  pipesd_model::Pending& p = model->pending;
  SeqState& s = p.kv->seqs[p.seq];
  const hipError_t e = hipStreamSynchronize(p.st);
  p.active = false;  // whatever happens next, the pass is over
  if (e != hipSuccess) {
    release_beyond(p.kv, s, p.text_len - 1);
    return hip_fail(e, "verify step");
  }
  if (layers_flag_raised(model)) {
    release_beyond(p.kv, s, p.text_len - 1);
    return hip_fail(hipErrorLaunchFailure, "device-wide barrier of the fused layer kernel timed out");
  }
  const int rc = commit_verify(model, p.kv, p.seq, p.drafts.data(), p.k, model->result_host, accepted_len, next_token);
  if (rc) release_beyond(p.kv, s, p.text_len - 1);
  return rc;
}

extern "C" int pipesd_nav_verify_chain(pipesd_model* model, pipesd_kv* kv, int32_t seq, int32_t prefix_len,
                                       int32_t n_rounds, const int32_t* k_per_round, const int32_t* tokens_concat,
                                       const float* const* draft_probs_per_round, const float* uniforms_concat,
                                       int32_t* accepted_len, int32_t* next_token, int32_t* rounds_run, void* stream) {
  if (!model || !kv || kv->model != model || !k_per_round || !tokens_concat || !accepted_len || !next_token ||
      !rounds_run)
    return PIPESD_EINVAL;
  if (n_rounds < 1 || n_rounds > 16 || !seq_ok(kv, seq)) return PIPESD_EINVAL;
  // ---- every check that can fail without running a pass comes before the first change of state ----
  std::vector<int32_t> tok_off(n_rounds), u_off(n_rounds);
  int32_t toks = 0, us = 0, growth = 0;
  for (int32_t r = 0; r < n_rounds; ++r) {
    const int32_t k = k_per_round[r];
    if (k < 1 || k > kMaxRows - 1) return PIPESD_EINVAL;
    if (r > 0) {  // the guess of the previous round's extra token
      if (tokens_concat[toks] < 0 || tokens_concat[toks] >= model->cfg.vocab) return PIPESD_EINVAL;
      ++toks;
    }
    tok_off[r] = toks;  // the round's drafts
    u_off[r] = us;
    toks += k;
    us += k + 1;
    growth += k + 1;
  }
  for (int pass = 0; pass < 2; ++pass)  // argument errors of every round first, then the state
    for (int32_t r = 0; r < (pass == 0 ? n_rounds : 1); ++r) {
      const float* qr = draft_probs_per_round ? draft_probs_per_round[r] : nullptr;
      const int rc = check_verify_args(model, kv, seq, prefix_len, tokens_concat + tok_off[r], k_per_round[r], qr,
                                       uniforms_concat ? uniforms_concat + u_off[r] : nullptr, pass == 1);
      if (rc) return rc;
    }
  {
    const SeqState& s = kv->seqs[seq];
    // the longest outcome: every round runs and accepts everything (the last round's rows included)
    const int64_t need = blocks_for((int32_t)s.text.size() - 1 + growth);
    if (need > (int64_t)s.blocks.size() + (int64_t)kv->free_list.size()) return PIPESD_ENOMEM;
  }
  *rounds_run = 0;
  hipStream_t st = (hipStream_t)stream;
  SeqState& s = kv->seqs[seq];
  if (model->cfg.dtype != PIPESD_BF16 || model->fused_enabled) {
    // one synchronisation per round: the rule is applied on the host between single calls
    int32_t lp = prefix_len;
    for (int32_t r = 0; r < n_rounds; ++r) {
      const int32_t k = k_per_round[r];
      if (r > 0) {  // Appendix B: the buffer survives iff all of round r-1 was accepted and the guess was right
        if (accepted_len[r - 1] != k_per_round[r - 1] || next_token[r - 1] != tokens_concat[tok_off[r] - 1]) break;
      }
      const float* qr = draft_probs_per_round ? draft_probs_per_round[r] : nullptr;
      const int rc = pipesd_nav_verify(model, kv, seq, lp, tokens_concat + tok_off[r], k, qr,
                                       uniforms_concat ? uniforms_concat + u_off[r] : nullptr, accepted_len + r,
                                       next_token + r, stream);
      if (rc) return rc;
      lp += accepted_len[r] + 1;
      *rounds_run = r + 1;
    }
    return PIPESD_OK;
  }
  // bf16: every round is enqueued at once and the rule is applied on the device.  Round r >= 1 is
  // enqueued for the state its buffer presumes (everything before it accepted, every guess right:
  // its rows, positions and blocks are then known on the host) and its launches are gated by a
  // device word that the step behind round r-1's decision sets: a round whose buffer turned out to
  // be invalid streams no weights and reports (-1, -1).  One synchronisation for the whole chain.
  const size_t text0 = s.text.size();
  auto give_up = [&]() {  // back to the state before the call
    s.text.resize(text0);
    release_beyond(kv, s, (int32_t)text0 - 1);
  };
  for (int32_t r = 0; r < n_rounds; ++r) model->result_host[4 + 2 * r] = model->result_host[4 + 2 * r + 1] = -1;
  int rc = PIPESD_OK;
  for (int32_t r = 0; r < n_rounds && rc == PIPESD_OK; ++r) {
    const int32_t k = k_per_round[r];
    const float* qr = draft_probs_per_round ? draft_probs_per_round[r] : nullptr;
    model->gate = r == 0 ? nullptr : model->chain_alive + r;
    rc = enqueue_verify(model, kv, seq, tokens_concat + tok_off[r], k, qr, uniforms_concat ? uniforms_concat + u_off[r] : nullptr,
                        model->result_dev + 2 * r, model->result_host + 4 + 2 * r, st);
    model->gate = nullptr;
    if (rc) break;
    const bool more = r + 1 < n_rounds;
    const hipError_t e = launch_chain_step(model->result_dev + 2 * r, model->result_host + 4 + 2 * r, k,
                                           more ? tokens_concat[tok_off[r + 1] - 1] : -1,
                                           r == 0 ? nullptr : model->chain_alive + r, more ? model->chain_alive + r + 1 : nullptr, st);
    if (e != hipSuccess) {
      rc = hip_fail(e, "chain step");
      break;
    }
    if (more) {  // the state round r + 1 presumes
      s.text.insert(s.text.end(), tokens_concat + tok_off[r], tokens_concat + tok_off[r] + k);
      s.text.push_back(tokens_concat[tok_off[r + 1] - 1]);
    }
  }
  const hipError_t es = hipStreamSynchronize(st);
  if (rc || es != hipSuccess) {
    give_up();
    return rc ? rc : hip_fail(es, "chained verify");
  }
  s.text.resize(text0);  // (the blocks reserved for the presumed states stay until the rounds are booked)
  // book the rounds that ran, one after the other, exactly as single calls would have
  for (int32_t r = 0; r < n_rounds; ++r) {
    const int32_t a = model->result_host[4 + 2 * r], nxt = model->result_host[4 + 2 * r + 1];
    if (r > 0 && (accepted_len[r - 1] != k_per_round[r - 1] || next_token[r - 1] != tokens_concat[tok_off[r] - 1])) {
      if (a != -1) return hip_fail(hipErrorLaunchFailure, "a round of the chain ran although its buffer was invalid");
      break;
    }
    // booking a round gives back the blocks beyond the rows it kept, those of later rounds included;
    // a later round that ran kept all rows before it, so its own blocks are reserved again (the free
    // list hands back the very blocks it was given last)
    rc = ensure_blocks(kv, seq, (int32_t)s.text.size() + k_per_round[r], st);
    if (rc == PIPESD_OK)
      rc = commit_verify(model, kv, seq, tokens_concat + tok_off[r], k_per_round[r], model->result_host + 4 + 2 * r,
                         accepted_len + r, next_token + r);
    if (rc) return rc;
    *rounds_run = r + 1;
  }
  return PIPESD_OK;
}

extern "C" int pipesd_nav_verify_batch(pipesd_model* model, pipesd_kv* kv, int32_t n_seqs, const int32_t* seq_ids,
                                       const int32_t* prefix_lens, const int32_t* k_per_seq,
                                       const int32_t* draft_tokens_concat, const float* const* draft_probs_per_seq,
                                       const float* uniforms_concat, int32_t* accepted_len, int32_t* next_token,
                                       void* stream) {
  if (!model || !kv || kv->model != model || !seq_ids || !prefix_lens || !k_per_seq || !draft_tokens_concat ||
      !accepted_len || !next_token)
    return PIPESD_EINVAL;
  if (n_seqs < 1 || n_seqs > kMaxBatch) return PIPESD_EINVAL;
  // ---- every check that can fail comes before the first change of state ----
  std::vector<int32_t> tok_off(n_seqs), u_off(n_seqs);
  int32_t toks = 0, us = 0;
  int64_t blocks_needed = 0;
  for (int32_t i = 0; i < n_seqs; ++i) {
    if (k_per_seq[i] < 1 || k_per_seq[i] > kMaxRows - 1) return PIPESD_EINVAL;
    tok_off[i] = toks;
    u_off[i] = us;
    toks += k_per_seq[i];
    us += k_per_seq[i] + 1;
  }
  for (int pass = 0; pass < 2; ++pass)  // argument errors of every client first, then states
    for (int32_t i = 0; i < n_seqs; ++i) {
      for (int32_t j = 0; j < i; ++j)
        if (seq_ids[j] == seq_ids[i]) return PIPESD_EINVAL;  // a sequence can take part once per call
      const float* qi = draft_probs_per_seq ? draft_probs_per_seq[i] : nullptr;
      int rc = check_verify_args(model, kv, seq_ids[i], prefix_lens[i], draft_tokens_concat + tok_off[i], k_per_seq[i],
                                 qi, uniforms_concat ? uniforms_concat + u_off[i] : nullptr, pass == 1);
      if (rc) return rc;
    }
  for (int32_t i = 0; i < n_seqs; ++i) {
    const SeqState& s = kv->seqs[seq_ids[i]];
    const int64_t need = blocks_for((int32_t)s.text.size() + k_per_seq[i]);
    if (need > (int64_t)s.blocks.size()) blocks_needed += need - (int64_t)s.blocks.size();
  }
  if (blocks_needed > (int64_t)kv->free_list.size()) return PIPESD_ENOMEM;
  // ---- enqueue sequence after sequence on the one stream, then wait once ----
  hipStream_t st = (hipStream_t)stream;
  auto undo = [&](int32_t upto) {
    for (int32_t i = 0; i < upto; ++i) {
      SeqState& s = kv->seqs[seq_ids[i]];
      release_beyond(kv, s, (int32_t)s.text.size() - 1);
    }
  };
  for (int32_t i = 0; i < 2 * n_seqs; ++i) model->result_host[4 + i] = -1;
  // bf16: clients are packed, in the order given, into passes of up to 256 rows and 16 clients, so
  // that the weights are streamed once per pass instead of once per client (a row's results do not
  // depend on which other rows share its pass); fp32: one pass per client
  const bool pack = model->cfg.dtype == PIPESD_BF16;
  for (int32_t first = 0; first < n_seqs;) {
    PassLayout pl;
    int32_t last = first;
    while (last < n_seqs && pl.n_clients < (pack ? kMaxPassClients : 1) &&
           pl.rows + k_per_seq[last] + 1 <= (pack ? kPassRowsCap : kMaxRows)) {
      const int32_t sq = seq_ids[last], k = k_per_seq[last];
      const SeqState& s = kv->seqs[sq];
      pl.client[pl.n_clients++] = PassClient{sq, k + 1, (int32_t)s.text.size() - 1};
      pl.tok.tok[pl.rows] = s.text.back();
      for (int32_t j = 0; j < k; ++j) pl.tok.tok[pl.rows + 1 + j] = draft_tokens_concat[tok_off[last] + j];
      pl.rows += k + 1;
      ++last;
    }
    int rc = PIPESD_OK;
    for (int32_t i = first; i < last && rc == PIPESD_OK; ++i)
      rc = ensure_blocks(kv, seq_ids[i], (int32_t)kv->seqs[seq_ids[i]].text.size() + k_per_seq[i], st);
    if (rc == PIPESD_OK) rc = run_pass(model, kv, pl, true, st);
    // The clients that use the sampling rule are decided, and their caches trimmed, by one launch
    // each for the whole pass (bf16, two or more such clients); token-matching clients, and passes
    // with a single sampling client, take the single-client kernels.
    int n_sampling = 0;
    for (int32_t i = first; i < last; ++i) n_sampling += (draft_probs_per_seq && draft_probs_per_seq[i]) ? 1 : 0;
    const bool batched = pack && n_sampling > 1;
    if (rc == PIPESD_OK && batched) {
      DecisionCall dc{};
      TrimBatch tb{};
      dc.logits = model->logits;
      dc.rows = pl.rows;
      dc.V = model->cfg.vocab;
      for (int32_t i = first, row_off = 0; i < last; ++i) {
        const int32_t k = k_per_seq[i];
        if (draft_probs_per_seq[i]) {
          dc.batch.c[dc.batch.n++] = DecisionClient{draft_probs_per_seq[i], row_off, k, i - first};
          for (int32_t j = 0; j < k; ++j) dc.batch.drafts.tok[row_off + j] = draft_tokens_concat[tok_off[i] + j];
          for (int32_t j = 0; j <= k; ++j) dc.batch.u[row_off + j] = uniforms_concat[u_off[i] + j];
          tb.c[tb.n++] = TrimClient{seq_ids[i] * kv->n_blocks, pl.client[i - first].start_pos, k, i - first};
        }
        row_off += k + 1;
      }
      dc.row_stats = model->row_stats;
      dc.scan_partial = model->scan_partial;
      dc.counter = model->counters + (kCounterSlots - 1 - kMaxPassClients);
      dc.result = model->result_dev + 2 * first;
      dc.result_copy = model->result_host + 4 + 2 * first;
      hipError_t e;
      {
        ProfScope ps(model, PIPESD_PROF_VERIFY, st);
        e = launch_spec_accept_batch(dc, st);
        if (e == hipSuccess)
          e = launch_kv_trim_batch(model->cfg.dtype, view_of(kv, 0), model->cfg.n_layers, tb, dc.result, st);
      }
      if (e != hipSuccess) rc = hip_fail(e, "batched verify");
    }
    for (int32_t i = first, row_off = 0; i < last && rc == PIPESD_OK; ++i) {
      const float* qi = draft_probs_per_seq ? draft_probs_per_seq[i] : nullptr;
      if (!(batched && qi)) {
        const hipError_t e = enqueue_decision(model, kv, seq_ids[i], row_off, pl.client[i - first].start_pos,
                                              draft_tokens_concat + tok_off[i], k_per_seq[i], qi,
                                              uniforms_concat ? uniforms_concat + u_off[i] : nullptr,
                                              model->result_dev + 2 * i, model->result_host + 4 + 2 * i, st);
        if (e != hipSuccess) rc = hip_fail(e, "batched verify");
      }
      row_off += k_per_seq[i] + 1;
    }
    if (rc) {
      (void)hipStreamSynchronize(st);
      undo(last);
      return rc;
    }
    first = last;
  }
  hipError_t e = read_layers_flag(model, st);
  if (e == hipSuccess) e = hipStreamSynchronize(st);
  if (e != hipSuccess) {
    undo(n_seqs);
    return hip_fail(e, "batched verify");
  }
  if (layers_flag_raised(model)) {
    undo(n_seqs);
    return hip_fail(hipErrorLaunchFailure, "device-wide barrier of the fused layer kernel timed out");
  }
  for (int32_t i = 0; i < n_seqs; ++i) {  // all decisions are checked before the first is booked
    const int32_t a = model->result_host[4 + 2 * i], nxt = model->result_host[4 + 2 * i + 1];
    if (a < 0 || a > k_per_seq[i] || nxt < 0 || nxt >= model->cfg.vocab) {
      undo(n_seqs);
      return PIPESD_EHIP;
    }
  }
  for (int32_t i = 0; i < n_seqs; ++i)
    (void)commit_verify(model, kv, seq_ids[i], draft_tokens_concat + tok_off[i], k_per_seq[i],
                        model->result_host + 4 + 2 * i, accepted_len + i, next_token + i);
  return PIPESD_OK;
}

extern "C" int pipesd_forward_logits(pipesd_model* model, pipesd_kv* kv, int32_t seq, const int32_t* tokens,
                                     int32_t n_extra, float* logits_out, void* stream) {
  if (!model || !kv || !logits_out || !seq_ok(kv, seq) || kv->model != model) return PIPESD_EINVAL;
  if (n_extra < 0 || n_extra > kMaxRows - 1 || (n_extra > 0 && !tokens)) return PIPESD_EINVAL;
  for (int32_t i = 0; i < n_extra; ++i)
    if (tokens[i] < 0 || tokens[i] >= model->cfg.vocab) return PIPESD_EINVAL;
  if (!compute_ready(model, kv)) return PIPESD_ESTATE;
  SeqState& s = kv->seqs[seq];
  const int32_t lp = (int32_t)s.text.size();
  if (lp < 1) return PIPESD_ESTATE;
  hipStream_t st = (hipStream_t)stream;
  int32_t start = 0;
  int rc = verify_common(model, kv, seq, tokens, n_extra, &start, st);
  if (rc) return rc;
  hipError_t e = hipMemcpyAsync(logits_out, model->logits, (size_t)(n_extra + 1) * model->cfg.vocab * 4,
                                hipMemcpyDeviceToHost, st);
  if (e == hipSuccess) e = read_layers_flag(model, st);
  if (e == hipSuccess) e = hipStreamSynchronize(st);
  release_beyond(kv, s, lp - 1);
  if (e == hipSuccess && layers_flag_raised(model))
    return hip_fail(hipErrorLaunchFailure, "device-wide barrier of the fused layer kernel timed out");
  return e == hipSuccess ? PIPESD_OK : hip_fail(e, "logits copy");
}

extern "C" int pipesd_spec_accept(const float* p, const float* q, const int32_t* draft_tokens, int32_t k, int32_t vocab,
                                  const float* uniforms, int32_t* accepted_len, int32_t* next_token, void* stream) {
  if (!p || !q || !draft_tokens || !uniforms || !accepted_len || !next_token) return PIPESD_EINVAL;
  if (k < 1 || k > kMaxRows - 1 || vocab < 1) return PIPESD_EINVAL;
  for (int32_t i = 0; i < k; ++i)
    if (draft_tokens[i] < 0 || draft_tokens[i] >= vocab) return PIPESD_EINVAL;
  for (int32_t i = 0; i <= k; ++i)
    if (!(uniforms[i] >= 0.f && uniforms[i] < 1.f)) return PIPESD_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  char* scratch = nullptr;
  HIP_TRY(hipMalloc((void**)&scratch, 4096));
  hipError_t e = hipMemsetAsync(scratch, 0, 4096, st);
  VerifyCall vc{};
  vc.logits_or_p = const_cast<float*>(p);
  vc.q = q;
  vc.k = k;
  vc.V = vocab;
  for (int32_t i = 0; i < k; ++i) vc.drafts.tok[i] = draft_tokens[i];
  for (int32_t i = 0; i <= k; ++i) vc.u[i] = uniforms[i];
  vc.scan_partial = (unsigned long long*)scratch;      // 64 x 8 bytes
  vc.counter = (unsigned*)(scratch + 1024);
  vc.result = (int32_t*)(scratch + 2048);
  int32_t host[2] = {-1, -1};
  if (e == hipSuccess) e = launch_spec_accept(vc, st);
  if (e == hipSuccess) e = hipMemcpyAsync(host, vc.result, 8, hipMemcpyDeviceToHost, st);
  if (e == hipSuccess) e = hipStreamSynchronize(st);
  (void)hipFree(scratch);
  if (e != hipSuccess) return hip_fail(e, "decision step");
  *accepted_len = host[0];
  *next_token = host[1];
  return PIPESD_OK;
}

// ---------------------------------------------------------------------------------------------
// Decision step for callers that cannot allocate: the scratch of the decision kernels (64 partial
// sums of the integer CDF, the arrival counter of its workgroups) lives in a file-scope device
// array.  The array's name is only a host-side stand-in; its device address is taken once per
// device with hipGetSymbolAddress and that pointer is what the kernels get.
// ---------------------------------------------------------------------------------------------
constexpr size_t kStaticScratchBytes = 4096;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kStaticMaxDevices = 64;
static void* g_static_scratch[kStaticMaxDevices] = {};

// device address of `scratch` on the current device (looked up on the first call on that device)
static int static_scratch_ptr(char** out) {
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kStaticMaxDevices) {
    snprintf(g_hip_msg, sizeof(g_hip_msg), "pipesd_spec_accept_static: device index %d beyond %d", dev, kStaticMaxDevices - 1);
    return PIPESD_EHIP;
  }
  if (g_static_scratch[dev] == nullptr) {
    void* ptr = nullptr;
    HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (ptr == nullptr) return hip_fail(hipErrorInvalidSymbol, "hipGetSymbolAddress(scratch)");
    g_static_scratch[dev] = ptr;
  }
  *out = (char*)g_static_scratch[dev];
  return PIPESD_OK;
}

extern "C" int pipesd_spec_accept_static(const float* p, const float* q, const int32_t* draft_tokens, int32_t k,
                                         int32_t vocab, const float* uniforms, int32_t* result_dev, void* stream) {
  if (!p || !q || !draft_tokens || !uniforms || !result_dev) return PIPESD_EINVAL;
  if (k < 1 || k > PIPESD_STATIC_MAX_K || vocab < 1 || vocab > PIPESD_STATIC_MAX_VOCAB) {
    snprintf(g_hip_msg, sizeof(g_hip_msg),
             "pipesd_spec_accept_static: k = %d, vocab = %d outside 1..%d drafts, 1..%d tokens (the static scratch is sized for these)",
             (int)k, (int)vocab, (int)PIPESD_STATIC_MAX_K, (int)PIPESD_STATIC_MAX_VOCAB);
    return PIPESD_EINVAL;
  }
  for (int32_t i = 0; i < k; ++i)
    if (draft_tokens[i] < 0 || draft_tokens[i] >= vocab) return PIPESD_EINVAL;
  for (int32_t i = 0; i <= k; ++i)
    if (!(uniforms[i] >= 0.f && uniforms[i] < 1.f)) return PIPESD_EINVAL;
  char* sp = nullptr;
  int rc = static_scratch_ptr(&sp);
  if (rc) return rc;
  hipStream_t st = (hipStream_t)stream;
  VerifyCall vc{};
  vc.logits_or_p = const_cast<float*>(p);
  vc.q = q;
  vc.k = k;
  vc.V = vocab;
  for (int32_t i = 0; i < k; ++i) vc.drafts.tok[i] = draft_tokens[i];
  for (int32_t i = 0; i <= k; ++i) vc.u[i] = uniforms[i];
  vc.scan_partial = (unsigned long long*)sp;  // 64 x 8 bytes
  vc.counter = (unsigned*)(sp + 1024);
  vc.result = result_dev;
  // the counter must start at zero whatever the call before left (a fill kernel, not a memset node:
  // the caller may be recording a graph)
  HIP_TRY(launch_clear_words(vc.counter, 1, st));
  HIP_TRY(launch_spec_accept(vc, st));
  return PIPESD_OK;
}

extern "C" int pipesd_kv_read(const pipesd_model* model, const pipesd_kv* kv, int32_t seq, int32_t layer, int32_t pos,
                              float* k_out, float* v_out) {
  if (!model || !kv || !k_out || !v_out || !seq_ok(kv, seq) || kv->model != model) return PIPESD_EINVAL;
  if (!compute_ready(model, kv)) return PIPESD_ESTATE;
  const pipesd_config& c = model->cfg;
  const SeqState& s = kv->seqs[seq];
  if (layer < 0 || layer >= c.n_layers || pos < 0 || pos / kBlockTokens >= (int32_t)s.blocks.size())
    return PIPESD_EINVAL;
  HIP_TRY(hipDeviceSynchronize());
  const size_t e = model->esz;
  const int h = c.head_dim, slot = pos % kBlockTokens;
  const int64_t base = (int64_t)layer * kv->layer_stride + (int64_t)s.blocks[pos / kBlockTokens] * kv->block_elems;
  std::vector<unsigned char> tk((size_t)h * e), tv((size_t)h * e);
  for (int kvh = 0; kvh < c.n_kv_heads; ++kvh) {
    const char* kp = (const char*)kv->pool + (base + ((int64_t)kvh * kBlockTokens + slot) * h) * e;
    const char* vp = (const char*)kv->pool + (base + kv->v_offset + (int64_t)kvh * h * kBlockTokens + slot) * e;
    HIP_TRY(hipMemcpy(tk.data(), kp, (size_t)h * e, hipMemcpyDeviceToHost));
    HIP_TRY(hipMemcpy2D(tv.data(), e, vp, (size_t)kBlockTokens * e, e, h, hipMemcpyDeviceToHost));
    for (int i = 0; i < h; ++i) {
      if (e == 4) {
        memcpy(&k_out[kvh * h + i], tk.data() + (size_t)i * 4, 4);
        memcpy(&v_out[kvh * h + i], tv.data() + (size_t)i * 4, 4);
      } else {
        uint16_t kb, vb;
        memcpy(&kb, tk.data() + (size_t)i * 2, 2);
        memcpy(&vb, tv.data() + (size_t)i * 2, 2);
        const uint32_t ku = (uint32_t)kb << 16, vu = (uint32_t)vb << 16;
        memcpy(&k_out[kvh * h + i], &ku, 4);
        memcpy(&v_out[kvh * h + i], &vu, 4);
      }
    }
  }
  return PIPESD_OK;
}
