// Device code of the bf16-cache attention of a NAV pass, shared by the per-layer attention kernels
// and the fused layer kernel.  (Masked self-attention of a decoder-only layer, Sec. 2.1; row r sees
// key positions 0..pos_r.)
//
// A wave loads 32 tokens' keys (two [16 tok][h] blocks, A operand of S^T = K Q^T) and values (two
// [h][16 tok] blocks, A operand of O^T = V^T P) straight from the paged cache in MFMA operand
// layout.  Queries and probabilities are fed as bf16 hi + lo pairs so only the cache itself is
// bf16.  The scores of one query row sit in the four lanes {c, c+16, c+32, c+48}, so the softmax
// statistics take two cross-lane steps.
//
// CO as in device_gemm.h: results other workgroups of the same kernel will read (partials, packed
// output) are written through; loads are ordinary cached loads.
#pragma once

#include "device_gemm.h"

namespace pipesd {

constexpr int kPartPad = 4;  // a partial row is [head_dim values, max, sum, 2 unused] so that rows stay 16-byte aligned
constexpr int kAttnWaves = 8;
constexpr int kAttnWgTokens = kAttnWaves * 32;

typedef __attribute__((ext_vector_type(4))) unsigned au32x4;
typedef __attribute__((ext_vector_type(2))) unsigned au32x2;

__device__ __forceinline__ void split_hi_lo8(const float (&v)[8], bf16x8& hi, bf16x8& lo) {
  unsigned h[4], l[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) split2_bf16(v[2 * i], v[2 * i + 1], h[i], l[i]);
  hi = __builtin_bit_cast(bf16x8, au32x4{h[0], h[1], h[2], h[3]});
  lo = __builtin_bit_cast(bf16x8, au32x4{l[0], l[1], l[2], l[3]});
}

// e^x through the hardware base-2 exponential (x <= 0 here; e^-inf = 0)
__device__ __forceinline__ float attn_exp(float x) { return __builtin_amdgcn_exp2f(x * 1.44269504088896341f); }
// n / m for 0 <= n < 4096, 1 <= m <= 128 with rinv = 1/m to within an ulp: (n + 0.5) / m is at least
// 0.5/m away from an integer, far more than the rounding error
__device__ __forceinline__ int div_small(int n, float rinv) { return (int)(((float)n + 0.5f) * rinv); }

constexpr size_t attn_lds_floats(int hd) { return (size_t)kAttnWaves * 16 * (hd + 4) + 2 * kAttnWaves * 16; }

// Task (kv_head, split, query tiles qt0..qt1-1) = 8 waves x 32 tokens against the query rows that
// share the KV head, 16 at a time (row rr of the head group is head kvh*group + rr/m, pass row
// rr%m).  Everything the task needs is requested up front (its keys, values and the first tile's
// queries; the next tile's queries while the current one is worked on); per tile each wave computes
// its 32 tokens' (max, sum, O), and after ONE workgroup barrier the eight results are merged by all
// 512 threads, waves in index order, and written as the split's partial.  A launch with few tasks
// gives every tile its own workgroup (shortest path); one with many lets a workgroup keep its keys
// and values in registers for all tiles.  The partials do not depend on that choice.  All 8 waves of
// the workgroup must call this together; the caller separates two calls on the same LDS by a barrier.
// MULTI = false: exactly one tile (qt1 is taken as qt0 + 1; fewer registers).
template <int HD, bool CO, bool MULTI = false>
__device__ __forceinline__ void attn_task(const float* q, const KvView& kv, int layer, int m, int start_pos,
                                          int n_q_heads, int nsplit, float* part, int kvh, int split, int qt0, int qt1,
                                          float* lds) {
  if constexpr (!MULTI) qt1 = qt0 + 1;
  constexpr int KSQ = HD / 32, HT = HD / 16, ROW = HD + 4;
  float(*o_lds)[16][ROW] = (float(*)[16][ROW])lds;
  float(*m_lds)[16] = (float(*)[16])(lds + (size_t)kAttnWaves * 16 * ROW);
  float(*l_lds)[16] = m_lds + kAttnWaves;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int c = lane & 15, g = lane >> 4;
  const int group = n_q_heads / kv.n_kv_heads;
  const int R = group * m;
  const int total = start_pos + m;
  const int tok0 = split * kAttnWgTokens + w * 32;
  const uint16_t* pool = (const uint16_t*)kv.pool;
  const float scale = 1.0f / sqrtf((float)HD);
  const float m_rinv = __builtin_amdgcn_rcpf((float)m);
  // all 32 tokens of this wave are cached tokens that every row of the pass sees: no masks needed
  const bool full = tok0 + 31 <= start_pos;

  // ---- requests: keys and values of this wave's 32 tokens, queries of row tile qt ----
  au32x4 kraw[2][KSQ];
  au32x2 vlo[HT], vhi[HT];
#pragma unroll
  for (int tt = 0; tt < 2; ++tt) {
    const int tb = tok0 + tt * 16;
    const int blk = kv.table[tb < total ? tb / kBlockTokens : 0];
    const int64_t base = (int64_t)layer * kv.layer_stride + (int64_t)blk * kv.block_elems;
#pragma unroll
    for (int s = 0; s < KSQ; ++s)
      kraw[tt][s] = *(const au32x4*)(pool + base + ((int64_t)kvh * kBlockTokens + c) * HD + s * 32 + g * 8);
#pragma unroll
    for (int j = 0; j < HT; ++j) {
      const au32x2 v = *(const au32x2*)(pool + base + kv.v_offset + ((int64_t)kvh * HD + j * 16 + c) * kBlockTokens + g * 4);
      if (tt == 0) vlo[j] = v; else vhi[j] = v;
    }
  }
  // queries arrive as bf16 hi + lo halves (written by the QKV epilogue): row = [n_q_heads*HD hi][.. lo]
  au32x4 qa[KSQ], qb[KSQ];  // hi, lo
  const uint16_t* q16 = (const uint16_t*)q;
  const int qd = n_q_heads * HD;
  auto q_request = [&](int qt) {  // rows beyond the head group read row 0 of the group (their results are dropped)
    const int rr = qt * 16 + c;
    const int gq = rr < R ? div_small(rr, m_rinv) : 0, r = rr < R ? rr - gq * m : 0;
#pragma unroll
    for (int s = 0; s < KSQ; ++s) {
      const uint16_t* qp = q16 + (size_t)r * 2 * qd + (kvh * group + gq) * HD + s * 32 + g * 8;
      qa[s] = *(const au32x4*)qp;
      qb[s] = *(const au32x4*)(qp + qd);
    }
  };
  q_request(qt0);

  // ---- operands: tokens at or beyond `total` read as zero ----
  bf16x8 kf[2][KSQ], vf[HT];
#pragma unroll
  for (int tt = 0; tt < 2; ++tt)
#pragma unroll
    for (int s = 0; s < KSQ; ++s) kf[tt][s] = __builtin_bit_cast(bf16x8, kraw[tt][s]);
#pragma unroll
  for (int j = 0; j < HT; ++j) vf[j] = __builtin_bit_cast(bf16x8, au32x4{vlo[j].x, vlo[j].y, vhi[j].x, vhi[j].y});
  if (!full) {
    unsigned long long keep[2];
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
      const int tb = tok0 + tt * 16;
      const bool tok_ok = tb + c < total;
#pragma unroll
      for (int s = 0; s < KSQ; ++s)
        kf[tt][s] = __builtin_bit_cast(bf16x8, tok_ok ? kraw[tt][s] : au32x4{0u, 0u, 0u, 0u});
      const int nvalid = min(4, max(0, total - (tb + g * 4)));
      keep[tt] = nvalid >= 4 ? ~0ull : ((1ull << (16 * nvalid)) - 1ull);
    }
#pragma unroll
    for (int j = 0; j < HT; ++j)
      vf[j] = __builtin_bit_cast(bf16x8, au32x4{vlo[j].x & (unsigned)keep[0], vlo[j].y & (unsigned)(keep[0] >> 32),
                                                vhi[j].x & (unsigned)keep[1], vhi[j].y & (unsigned)(keep[1] >> 32)});
  }
  for (int qt = qt0; qt < qt1; ++qt) {
  const int rr = qt * 16 + c;
  const int r = rr < R ? rr - div_small(rr, m_rinv) * m : 0;
  bf16x8 qhi[KSQ], qlo[KSQ];
#pragma unroll
  for (int s = 0; s < KSQ; ++s) {
    qhi[s] = __builtin_bit_cast(bf16x8, qa[s]);
    qlo[s] = __builtin_bit_cast(bf16x8, qb[s]);
  }

  // ---- scores of query row c against tokens tok0 + tt*16 + g*4 + i ----
  float sc[8];
  const int pos_q = start_pos + r;
#pragma unroll
  for (int tt = 0; tt < 2; ++tt) {
    f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < KSQ; ++s) {
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[tt][s], qhi[s], acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[tt][s], qlo[s], acc, 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) sc[tt * 4 + i] = acc[i] * scale;
  }
  if (!full) {
#pragma unroll
    for (int i = 0; i < 8; ++i)
      if (tok0 + (i >> 2) * 16 + g * 4 + (i & 3) > pos_q) sc[i] = -INFINITY;
  }
  float m_run = sc[0];
#pragma unroll
  for (int i = 1; i < 8; ++i) m_run = fmaxf(m_run, sc[i]);
  m_run = fmaxf(m_run, __shfl_xor(m_run, 16, 64));
  m_run = fmaxf(m_run, __shfl_xor(m_run, 32, 64));
  const float m_ref = (m_run == -INFINITY) ? 0.f : m_run;  // a row that sees none of the tokens: all weights 0
  float pv[8], l_run = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    pv[i] = attn_exp(sc[i] - m_ref);
    l_run += pv[i];
  }
  l_run += __shfl_xor(l_run, 16, 64);
  l_run += __shfl_xor(l_run, 32, 64);
  bf16x8 phi, plo;
  split_hi_lo8(pv, phi, plo);
#pragma unroll
  for (int j = 0; j < HT; ++j) {
    f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[j], phi, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[j], plo, acc, 0, 0, 0);
    *(f32x4*)&o_lds[w][c][j * 16 + g * 4] = acc;  // O[query c][element j*16 + g*4 + i]
  }
  if (g == 0) {
    m_lds[w][c] = m_run;
    l_lds[w][c] = l_run;
  }
  __syncthreads();
  if (qt + 1 < qt1) q_request(qt + 1);  // travels during the merge

  // ---- merge of the eight waves: thread -> (query row, 4 consecutive elements), waves in index order ----
  constexpr int TPR = HD / 4;  // threads per row: all 512 threads for h = 128, the first 256 for h = 64
  const int mr = tid / TPR, e0 = (tid % TPR) * 4;
  if (mr < 16) {
    float M = m_lds[0][mr];
#pragma unroll
    for (int ww = 1; ww < kAttnWaves; ++ww) M = fmaxf(M, m_lds[ww][mr]);
    const float M_ref = (M == -INFINITY) ? 0.f : M;
    float L = 0.f;
    f32x4 o = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ww = 0; ww < kAttnWaves; ++ww) {
      const float sw = attn_exp(m_lds[ww][mr] - M_ref);
      L += l_lds[ww][mr] * sw;
      o += *(const f32x4*)&o_lds[ww][mr][e0] * sw;
    }
    const int rr2 = qt * 16 + mr;
    if (rr2 < R) {
      const int g2 = div_small(rr2, m_rinv);
      const int head2 = kvh * group + g2, r2 = rr2 - g2 * m;
      float* dst = part + (((size_t)head2 * m + r2) * nsplit + split) * (HD + kPartPad);
      Xwg<CO>::st4f(dst + e0, o);
      if (e0 == 0) Xwg<CO>::st4f(dst + HD, f32x4{M, L, 0.f, 0.f});
    }
  }
  if (qt + 1 < qt1) __syncthreads();  // the merge has read the LDS the next tile writes
  }
}

// Merge the splits of one (row, head) for 8 consecutive elements e0..e0+7: o = sum_s e^{m_s - M} o_s /
// sum_s e^{m_s - M} l_s, splits taken in index order, all of a batch's loads issued before any is
// used.  `row_of(s)` points at split s's partial row [h values, max, sum, 2 unused].
template <typename RowOf>
__device__ __forceinline__ void attn_merge_rows(RowOf row_of, int nsplit, int h, int e0, float (&acc)[8]) {
  constexpr int BATCH = 9;
  float M = -INFINITY, L = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = 0.f;
  for (int s0 = 0; s0 < nsplit; s0 += BATCH) {
    au32x4 mlr[BATCH], oar[BATCH], obr[BATCH];
#pragma unroll
    for (int j = 0; j < BATCH; ++j) {
      const float* ps = row_of(min(s0 + j, nsplit - 1));
      mlr[j] = *(const au32x4*)(ps + h);
      oar[j] = *(const au32x4*)(ps + e0);
      obr[j] = *(const au32x4*)(ps + e0 + 4);
    }
    f32x4 ml[BATCH], oa[BATCH], ob[BATCH];
#pragma unroll
    for (int j = 0; j < BATCH; ++j) {
      ml[j] = __builtin_bit_cast(f32x4, mlr[j]);
      oa[j] = __builtin_bit_cast(f32x4, oar[j]);
      ob[j] = __builtin_bit_cast(f32x4, obr[j]);
    }
    float bm = M;
#pragma unroll
    for (int j = 0; j < BATCH; ++j)
      if (s0 + j < nsplit) bm = fmaxf(bm, ml[j][0]);
    if (bm == -INFINITY) continue;
    const float so = (M == -INFINITY) ? 0.f : attn_exp(M - bm);
    L *= so;
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] *= so;
#pragma unroll
    for (int j = 0; j < BATCH; ++j) {
      const float wgt = (s0 + j < nsplit && ml[j][0] != -INFINITY) ? attn_exp(ml[j][0] - bm) : 0.f;
      L += ml[j][1] * wgt;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        acc[i] += oa[j][i] * wgt;
        acc[i + 4] += ob[j][i] * wgt;
      }
    }
    M = bm;
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] /= L;
}

// One thread of the merge of a pass's partials [(head*m + r)*nsplit + split][h + 4]; the result is
// written packed for the O projection.  `gt` numbers the threads over all (pair, segment) tasks.
// `row_off`: the client's first row in the pass (rows of the packed output).
template <bool CO>
__device__ __forceinline__ void attn_merge_thread(const float* part, int m, int n_q_heads, int h, int nsplit,
                                                  u32x4* outp, int gt, int row_off = 0, int act_tiles = 2) {
  const int segs = h / 8;
  const int pair = gt / segs, e0 = (gt % segs) * 8;  // pair = head * m + r
  if (pair >= m * n_q_heads) return;
  const int head = pair / m, r = pair % m;
  const float* p = part + (size_t)pair * nsplit * (h + kPartPad);
  float acc[8];
  attn_merge_rows([&](int s) { return p + (size_t)s * (h + kPartPad); }, nsplit, h, e0, acc);
  store_act8x<CO>(outp, row_off + r, head * h + e0, acc, act_tiles);
}

}  // namespace pipesd
