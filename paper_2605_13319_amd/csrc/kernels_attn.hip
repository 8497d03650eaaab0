// Grouped-query attention of the m = k + 1 causal rows of a pass over the paged KV cache.
// (Masked self-attention of a decoder-only layer, Sec. 2.1; row r sees key positions 0..pos_r.)
//
// Split over the context: workgroup (kv_head, split) handles `chunk` consecutive tokens for every
// query row of the query heads that share the KV head, producing an un-normalised partial
// (max, sum, o); a second kernel merges the splits in a fixed order, so results do not depend on
// scheduling.
#include <algorithm>

#include "device_attn.h"
#include "device_dma.h"

namespace pipesd {

constexpr int kAttnThreads = 256;
constexpr int kAttnChunkMax = 32;

template <typename T>
__global__ __launch_bounds__(kAttnThreads) void attn_partial_kernel(const float* __restrict__ q, KvView kv, int layer,
                                                                    int m, int start_pos, int n_q_heads, int chunk,
                                                                    int nsplit, float* __restrict__ part) {
  extern __shared__ float lds[];
  const int h = kv.head_dim;
  const int hp = h + 1;
  float* ks = lds;                          // [chunk][h+1]
  float* vs = ks + kAttnChunkMax * hp;      // [chunk][h+1]
  float* qs = vs + kAttnChunkMax * hp;      // [m][h]
  float* ps = qs + kMaxRows * h;            // [m][chunk]
  const int kvh = blockIdx.x, split = blockIdx.y;
  const int group = n_q_heads / kv.n_kv_heads;
  const int total = start_pos + m;          // keys visible to the last row
  const int t0 = split * chunk;
  const int nt = min(chunk, total - t0);
  const int tid = threadIdx.x;
  const T* pool = (const T*)kv.pool;
  const float scale = 1.0f / sqrtf((float)h);

  for (int i = tid; i < nt * h; i += kAttnThreads) {
    const int t = i / h, e = i % h;
    ks[t * hp + e] = load_elem(pool, k_index(kv, layer, t0 + t, kvh, e));
  }
  for (int i = tid; i < nt * h; i += kAttnThreads) {
    const int e = i / nt, t = i % nt;  // the value block keeps tokens contiguous per element
    vs[t * hp + e] = load_elem(pool, v_index(kv, layer, t0 + t, kvh, e));
  }

  for (int gq = 0; gq < group; ++gq) {
    const int head = kvh * group + gq;
    __syncthreads();
    for (int i = tid; i < m * h; i += kAttnThreads) {
      const int r = i / h, e = i % h;
      qs[i] = q[((size_t)r * n_q_heads + head) * h + e];
    }
    __syncthreads();
    // scores
    for (int i = tid; i < m * chunk; i += kAttnThreads) {
      const int r = i / chunk, t = i % chunk;
      float s = -INFINITY;
      if (t < nt && t0 + t <= start_pos + r) {
        float acc = 0.f;
        for (int e = 0; e < h; ++e) acc = fmaf(qs[r * h + e], ks[t * hp + e], acc);
        s = acc * scale;
      }
      ps[i] = s;
    }
    __syncthreads();
    // per row: max, exp, sum (one thread per row; rows and chunk are small)
    if (tid < m) {
      float mx = -INFINITY;
      for (int t = 0; t < chunk; ++t) mx = fmaxf(mx, ps[tid * chunk + t]);
      float l = 0.f;
      for (int t = 0; t < chunk; ++t) {
        const float s = ps[tid * chunk + t];
        const float p = (s == -INFINITY) ? 0.f : expf(s - mx);
        ps[tid * chunk + t] = p;
        l += p;
      }
      float* o = part + (((size_t)head * m + tid) * nsplit + split) * (h + kPartPad);
      o[h] = mx;
      o[h + 1] = l;
    }
    __syncthreads();
    // o = P V
    for (int i = tid; i < m * h; i += kAttnThreads) {
      const int r = i / h, e = i % h;
      float acc = 0.f;
      for (int t = 0; t < nt; ++t) acc = fmaf(ps[r * chunk + t], vs[t * hp + e], acc);
      part[(((size_t)head * m + r) * nsplit + split) * (h + kPartPad) + e] = acc;
    }
  }
}

// ------------------------------------------------------------------------------------------------
// bf16 cache: the same computation on the matrix cores (device code in device_attn.h)
// ------------------------------------------------------------------------------------------------
// grid = (kv heads, splits of all clients of the pass one client after the other, query tiles of the
// largest client / qpw); a workgroup takes qpw query tiles (MULTI) or one
template <int HD, bool MULTI>
__global__ __launch_bounds__(kAttnWaves * 64) void attn_mfma_kernel(const float* q, KvView kv, int layer, int n_q_heads,
                                                                    AttnBatch batch, float* part, int qpw,
                                                                    const int32_t* gate) {
  extern __shared__ float lds[];
  if (gate != nullptr && *gate == 0) return;  // (uniform: a round of a chain that does not run)
  const int kvh = blockIdx.x;
  int ci = 0, split = blockIdx.y;
  while (ci + 1 < batch.n && split >= batch.c[ci].nsplit) split -= batch.c[ci++].nsplit;
  const AttnClient c = batch.c[ci];
  const int nqt = (n_q_heads / kv.n_kv_heads * c.m + 15) / 16, qt0 = (int)blockIdx.z * qpw;
  if (split >= c.nsplit || qt0 >= nqt) return;  // whole workgroup
  kv.table += c.table_off;
  attn_task<HD, false, MULTI>(q + (size_t)c.row_off * n_q_heads * HD, kv, layer, c.m, c.start_pos, n_q_heads,
                              c.nsplit, part + c.part_off, kvh, split, qt0, min(nqt, qt0 + qpw), lds);
}

// ------------------------------------------------------------------------------------------------
// bf16 cache, passes of few rows per client (the NAV pass itself) and prompt blocks: one workgroup
// walks a whole split of the context
// ------------------------------------------------------------------------------------------------
// Workgroup (kv head, split of a client's context, T query tiles) of four waves: wave w takes tokens
// span0 + it*128 + w*32 .. + 31 in step it and keeps a running (max, sum, O) per query tile in
// registers.  A step's keys are requested one step ahead, into registers.  So are its values for
// T = 1; for T = 2 (twice the running state, no registers left for that) the values of the next
// step are copied from memory straight into an LDS buffer of the wave's own (the LDS its state goes
// to in the merge) as soon as the wave has read the current step's out of it, and travel during the
// rest of the step and the next step's scores.  After the last step the four waves' states are
// merged through LDS, waves in index order.  A client whose
// context is one split gets its normalised rows written straight in the packed form the O
// projection reads.  Otherwise the workgroup writes its partial through to memory and counts
// itself in; the workgroup that arrives last merges the splits, in index order, and writes the
// packed rows: no second launch.  The queries of the workgroup's tiles sit in LDS in operand order
// (hi and lo halves), read again in every step.  What a row's result is depends on the client's own
// context and rows only, never on the other clients of the pass, on T or on which workgroup came last.
//
// Partials: per (client, kv head, tile group) [split][T tiles][16 rows][HD + 4] floats, each
// [split] block a whole number of 128-byte lines, so no cache line holds partials of two groups:
// the merging workgroup reads lines nobody on its compute unit has touched during this kernel,
// after every writer has drained its write-through stores and then incremented the counter.
constexpr int kStreamWaves = 4;                // waves per workgroup: one per SIMD, so that two workgroups in different
                                               // phases (waiting for keys and values / multiplying) share a compute unit
constexpr int kStreamWgTokens = kStreamWaves * 32;  // tokens per workgroup and step
constexpr int kStreamMaxSteps = 64;            // steps of a split (a lane per step holds its block-table entries)
constexpr int kStreamMinSpan = 256;            // a client's context is cut into at most kStreamMaxSplits
constexpr int kStreamMaxSplits = 16;           // splits of 256 * 2^j tokens, j as small as that allows
constexpr int kStreamMaxRows = 128;            // rows of a client (a prompt block brings up to 128; a NAV pass at most kMaxRows)

constexpr size_t stream_lds_floats(int hd) { return (size_t)kStreamWaves * 16 * (hd + 4) + 2 * kStreamWaves * 16; }
template <int HD>
constexpr size_t stream_lds_bytes(int T) {
  return stream_lds_floats(HD) * sizeof(float) + (size_t)T * (HD / 32) * 2 * 64 * 16 + 16;
}

template <int HD, int T>
__global__ __launch_bounds__(kStreamWaves * 64, 2) void attn_stream_kernel(const float* q, KvView kv, int layer, int n_q_heads,
                                                                      AttnBatch batch, float* part, uint4* outp,
                                                                      int act_tiles, const int32_t* gate,
                                                                      unsigned* counters) {
  extern __shared__ float lds[];
  if (gate != nullptr && *gate == 0) return;  // (uniform: a round of a chain that does not run)
  constexpr int KSQ = HD / 32, HT = HD / 16, ROW = HD + 4;
  const int kvh = blockIdx.x;
  int ci = 0, split = blockIdx.y;
  while (ci + 1 < batch.n && split >= batch.c[ci].nsplit) split -= batch.c[ci++].nsplit;
  const AttnClient cl = batch.c[ci];
  const int group = n_q_heads / kv.n_kv_heads, m = cl.m, R = group * m;
  const int nqt = (R + 15) / 16, qt0 = (int)blockIdx.z * T;
  if (split >= cl.nsplit || qt0 >= nqt) return;  // whole workgroup
  float(*o_lds)[16][ROW] = (float(*)[16][ROW])lds;
  float(*m_lds)[16] = (float(*)[16])(lds + (size_t)kStreamWaves * 16 * ROW);
  float(*l_lds)[16] = m_lds + kStreamWaves;
  au32x4* q_lds = (au32x4*)(lds + stream_lds_floats(HD));  // [T][KSQ][hi, lo][64 lanes]
  int* last_lds = (int*)(q_lds + T * KSQ * 2 * 64);
  const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int c = lane & 15, g = lane >> 4;
  const int total = cl.start_pos + m;
  const int span0 = split * cl.span, span1 = min(total, span0 + cl.span);
  const int nsteps = (span1 - span0 + kStreamWgTokens - 1) / kStreamWgTokens;
  const uint16_t* pool = (const uint16_t*)kv.pool;
  const int32_t* table = kv.table + cl.table_off;
  const float scale = 1.0f / sqrtf((float)HD);
  const float m_rinv = __builtin_amdgcn_rcpf((float)m);
  const int qd = n_q_heads * HD;

  // ---- queries of the T tiles: global (row = [qd hi halves][qd lo halves]) -> LDS in operand order ----
  constexpr int QCH = 16 * (HD / 8) * 2;  // 16-byte pieces per tile
  constexpr int QPT = (QCH + kStreamWaves * 64 - 1) / (kStreamWaves * 64);  // pieces per thread and tile
  au32x4 qreg[T][QPT];
  {
    const uint16_t* q16 = (const uint16_t*)q + (size_t)cl.row_off * 2 * qd;
#pragma unroll
    for (int i = 0; i < QPT; ++i) {
      const int piece = tid + i * kStreamWaves * 64;
      const int hl = piece / (16 * (HD / 8)), rem = piece % (16 * (HD / 8)), qc = rem / (HD / 8), j = rem % (HD / 8);
#pragma unroll
      for (int t = 0; t < T; ++t) {
        const int rr = (qt0 + t) * 16 + qc;  // rows beyond the head group read row 0 of the group (their results are dropped)
        const int gq = rr < R ? div_small(rr, m_rinv) : 0, r = rr < R ? rr - gq * m : 0;
        qreg[t][i] = piece < QCH ? *(const au32x4*)(q16 + (size_t)r * 2 * qd + hl * qd + (kvh * group + gq) * HD + j * 8)
                                 : au32x4{0u, 0u, 0u, 0u};
      }
    }
  }

  struct KRegs {
    au32x4 k[2][KSQ];
  };
  struct VRegs {
    au32x2 lo[HT], hi[HT];
  };
  // The block-table entries of this wave's tokens are read once, before the first step, and held in
  // registers: lane L has the two of step L (a split is at most 64 steps).  Looked up from memory
  // per request, every request would first wait for all loads before it, the step's keys and
  // values among them.
  int step_blk[2];
#pragma unroll
  for (int tt = 0; tt < 2; ++tt) {
    const int tb = span0 + lane * kStreamWgTokens + w * 32 + tt * 16;
    step_blk[tt] = table[tb < total ? tb / kBlockTokens : 0];
  }
  auto block_base = [&](int it, int tt) {
    const int blk = __builtin_amdgcn_readlane(step_blk[tt], it);
    return (int64_t)layer * kv.layer_stride + (int64_t)blk * kv.block_elems;
  };
  auto request_k = [&](KRegs& b, int it) {
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
      const int64_t base = block_base(it, tt);
#pragma unroll
      for (int s = 0; s < KSQ; ++s)
        b.k[tt][s] = *(const au32x4*)(pool + base + ((int64_t)kvh * kBlockTokens + c) * HD + s * 32 + g * 8);
    }
  };
  auto request_v = [&](VRegs& b, int it) {
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
      const int64_t base = block_base(it, tt);
#pragma unroll
      for (int j = 0; j < HT; ++j) {
        const au32x2 v = *(const au32x2*)(pool + base + kv.v_offset + ((int64_t)kvh * HD + j * 16 + c) * kBlockTokens + g * 4);
        if (tt == 0) b.lo[j] = v; else b.hi[j] = v;
      }
    }
  };

  // T = 2: the values of a step through LDS.  The wave's buffer holds the step's two blocks as they
  // are in memory ([element][16 tokens]); one load instruction copies 32 elements' rows (lane ->
  // element lane/2, tokens 8 (lane&1) .. +7).
  constexpr int NVL = 2 * (HD / 32);  // load instructions per step
  char* vbuf = (char*)lds + (size_t)w * 16 * ROW * sizeof(float);  // (= the wave's rows of o_lds)
  static_assert(2 * HD * kBlockTokens * 2 <= 16 * ROW * (int)sizeof(float), "a step's values fit the wave's merge rows");
  auto request_v_lds = [&](int it) {
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
      const int64_t base = block_base(it, tt);
#pragma unroll
      for (int qd32 = 0; qd32 < HD / 32; ++qd32) {
        const uint16_t* src = pool + base + kv.v_offset + ((int64_t)kvh * HD + qd32 * 32 + (lane >> 1)) * kBlockTokens + (lane & 1) * 8;
        lds_dma16(src, vbuf + (tt * (HD / 32) + qd32) * 1024);
      }
    }
  };

  // running state per tile: scores of query row c sit in lanes {c, c+16, c+32, c+48}, and so do the
  // statistics and (as O^T) the outputs of that row
  float m_run[T], l_run[T];
  f32x4 oacc[T][HT];
  int pos_q[T];
#pragma unroll
  for (int t = 0; t < T; ++t) {
    m_run[t] = -INFINITY;
    l_run[t] = 0.f;
#pragma unroll
    for (int j = 0; j < HT; ++j) oacc[t][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    const int rr = (qt0 + t) * 16 + c;
    pos_q[t] = cl.start_pos + (rr < R ? rr - div_small(rr, m_rinv) * m : 0);
  }

  // T = 1: keys and values of a step are both requested a step ahead, into registers.  T = 2: the
  // keys are; the values come through the wave's LDS buffer.  This wave's vector-memory operations
  // complete in the order issued, and the order is: keys 0, values 0, keys 1 (all landed before
  // step 0) | step 0: values 1, keys 2 | step 1: values 2, keys 3 | ..  So a step's values have
  // landed once at most the loads of the next step's keys (if there is a next step) are outstanding.
  constexpr bool V_AHEAD = T == 1;
  auto consume = [&](const KRegs& bk, VRegs& bv, int it) {
    const int tok0 = span0 + it * kStreamWgTokens + w * 32;
    if (tok0 >= total) return;  // (wave-uniform) nothing cached there
    asm volatile("" ::: "memory");  // the queries are read from LDS in every step, not kept in registers
    // all 32 tokens are cached tokens that every row of the pass sees: no masks needed
    const bool full = tok0 + 31 <= cl.start_pos;
    bf16x8 kf[2][KSQ], vf[HT];
#pragma unroll
    for (int tt = 0; tt < 2; ++tt)
#pragma unroll
      for (int s = 0; s < KSQ; ++s) kf[tt][s] = __builtin_bit_cast(bf16x8, bk.k[tt][s]);
    if constexpr (V_AHEAD) {
#pragma unroll
      for (int j = 0; j < HT; ++j) vf[j] = __builtin_bit_cast(bf16x8, au32x4{bv.lo[j].x, bv.lo[j].y, bv.hi[j].x, bv.hi[j].y});
    } else {
      if (it + 1 < nsteps)
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * KSQ) : "memory");
      else
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
      for (int j = 0; j < HT; ++j) {
        const au32x2 lo = *(const au32x2*)(vbuf + (j * 16 + c) * (kBlockTokens * 2) + g * 8);
        const au32x2 hi = *(const au32x2*)(vbuf + HD * kBlockTokens * 2 + (j * 16 + c) * (kBlockTokens * 2) + g * 8);
        vf[j] = __builtin_bit_cast(bf16x8, au32x4{lo.x, lo.y, hi.x, hi.y});
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the buffer has been read: it can take the next step's values
    }
    if (!full) {
      // values of tokens at or beyond `total` read as zero (their weights are exact zeros, but what the
      // cache holds there need not be a number); their keys need nothing: those scores are masked below
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
        const int nvalid = min(4, max(0, total - (tok0 + tt * 16 + g * 4)));
        const unsigned long long keep = nvalid >= 4 ? ~0ull : ((1ull << (16 * nvalid)) - 1ull);
        const unsigned k0 = (unsigned)keep, k1 = (unsigned)(keep >> 32);
#pragma unroll
        for (int j = 0; j < HT; ++j) {
          au32x4 v = __builtin_bit_cast(au32x4, vf[j]);
          if (tt == 0) { v.x &= k0; v.y &= k1; } else { v.z &= k0; v.w &= k1; }
          vf[j] = __builtin_bit_cast(bf16x8, v);
        }
      }
    }
#pragma unroll
    for (int t = 0; t < T; ++t) {
      if (qt0 + t >= nqt) break;  // (workgroup-uniform)
      float sc[8];
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
        f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < KSQ; ++s) {
          const bf16x8 qhi = __builtin_bit_cast(bf16x8, q_lds[((t * KSQ + s) * 2 + 0) * 64 + lane]);
          const bf16x8 qlo = __builtin_bit_cast(bf16x8, q_lds[((t * KSQ + s) * 2 + 1) * 64 + lane]);
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[tt][s], qhi, acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[tt][s], qlo, acc, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) sc[tt * 4 + i] = acc[i] * scale;
      }
      if constexpr (!V_AHEAD) {
        // The next step's values are asked for here, behind the first tile's scores: every key
        // fragment of the step has been used by now, so the compiler's waits for them, which do not
        // count these copies, have all been passed and none of them ends up waiting for the copies.
        // (Asked for without a branch, which would put a block boundary between the multiplies and
        // the first use of their results: the last step asks for its own values again, never read.)
        if (t == 0) {
          __builtin_amdgcn_sched_barrier(0);
          request_v_lds(min(it + 1, nsteps - 1));
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      if (!full) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
          if (tok0 + (i >> 2) * 16 + g * 4 + (i & 3) > pos_q[t]) sc[i] = -INFINITY;
      }
      float m_new = sc[0];
#pragma unroll
      for (int i = 1; i < 8; ++i) m_new = fmaxf(m_new, sc[i]);
      m_new = fmaxf(m_new, __shfl_xor(m_new, 16, 64));
      m_new = fmaxf(m_new, __shfl_xor(m_new, 32, 64));
      m_new = fmaxf(m_new, m_run[t]);
      const float m_ref = (m_new == -INFINITY) ? 0.f : m_new;  // a row that has seen no token yet: all weights 0
      const float alpha = attn_exp(m_run[t] - m_ref);          // e^-inf = 0 for the first tokens a row sees
      float pv[8], l_step = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        pv[i] = attn_exp(sc[i] - m_ref);
        l_step += pv[i];
      }
      l_step += __shfl_xor(l_step, 16, 64);
      l_step += __shfl_xor(l_step, 32, 64);
      l_run[t] = l_run[t] * alpha + l_step;
      m_run[t] = m_new;
      bf16x8 phi, plo;
      split_hi_lo8(pv, phi, plo);
#pragma unroll
      for (int j = 0; j < HT; ++j) {
        f32x4 acc = oacc[t][j] * alpha;
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[j], phi, acc, 0, 0, 0);
        oacc[t][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[j], plo, acc, 0, 0, 0);
      }
    }
  };

  KRegs ka, kb;
  VRegs va, vb;
  request_k(ka, 0);
  if constexpr (V_AHEAD) request_v(va, 0); else request_v_lds(0);
  if (nsteps > 1) {
    request_k(kb, 1);
    if constexpr (V_AHEAD) request_v(vb, 1);
  }
#pragma unroll
  for (int i = 0; i < QPT; ++i) {
    const int piece = tid + i * kStreamWaves * 64;
    const int hl = piece / (16 * (HD / 8)), rem = piece % (16 * (HD / 8)), qc = rem / (HD / 8), j = rem % (HD / 8);
    if (piece < QCH) {
#pragma unroll
      for (int t = 0; t < T; ++t) q_lds[((t * KSQ + (j >> 2)) * 2 + hl) * 64 + (j & 3) * 16 + qc] = qreg[t][i];
    }
  }
  __syncthreads();
  for (int it = 0; it < nsteps; it += 2) {
    consume(ka, va, it);
    if (it + 2 < nsteps) {
      request_k(ka, it + 2);
      if constexpr (V_AHEAD) request_v(va, it + 2);
    }
    if (it + 1 < nsteps) {
      consume(kb, V_AHEAD ? vb : va, it + 1);
      if (it + 3 < nsteps) {
        request_k(kb, it + 3);
        if constexpr (V_AHEAD) request_v(vb, it + 3);
      }
    }
  }

  // (T = 2: a wave that found nothing cached in its last steps never waited for the values it had
  // requested; they must have landed before its merge rows, the same LDS, are written)
  if constexpr (!V_AHEAD) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  // (The last products may have been issued in another basic block, where the compiler pads too few
  // wait states for the LDS stores of their results below: spell them out.)
  __builtin_amdgcn_sched_barrier(0);
  asm volatile("s_nop 15\n\ts_nop 7" ::: "memory");
  __builtin_amdgcn_sched_barrier(0);

  // ---- merge of the waves, tile after tile: thread -> (query row, 8 consecutive elements) ----
  constexpr int TPR = HD / 8;
  const int mr = tid / TPR, e0 = (tid % TPR) * 8;
  const int nz = (nqt + T - 1) / T;
  float* gpart = part + cl.part_off + (size_t)(kvh * nz + (int)blockIdx.z) * cl.nsplit * (T * 16 * ROW);
#pragma unroll
  for (int t = 0; t < T; ++t) {
    if (qt0 + t >= nqt) break;
    if (t > 0) __syncthreads();  // the merge of the tile before has read the LDS this tile writes
#pragma unroll
    for (int j = 0; j < HT; ++j) *(f32x4*)&o_lds[w][c][j * 16 + g * 4] = oacc[t][j];  // O[query c][element j*16 + g*4 + i]
    if (g == 0) {
      m_lds[w][c] = m_run[t];
      l_lds[w][c] = l_run[t];
    }
    __syncthreads();
    if (mr < 16) {
      float M = m_lds[0][mr];
#pragma unroll
      for (int ww = 1; ww < kStreamWaves; ++ww) M = fmaxf(M, m_lds[ww][mr]);
      const float M_ref = (M == -INFINITY) ? 0.f : M;
      float L = 0.f;
      f32x4 oa = f32x4{0.f, 0.f, 0.f, 0.f}, ob = oa;
#pragma unroll
      for (int ww = 0; ww < kStreamWaves; ++ww) {
        const float sw = attn_exp(m_lds[ww][mr] - M_ref);
        L += l_lds[ww][mr] * sw;
        oa += *(const f32x4*)&o_lds[ww][mr][e0] * sw;
        ob += *(const f32x4*)&o_lds[ww][mr][e0 + 4] * sw;
      }
      const int rr2 = (qt0 + t) * 16 + mr;
      if (rr2 < R) {
        if (cl.nsplit == 1) {
          const int g2 = div_small(rr2, m_rinv);
          const int head2 = kvh * group + g2, r2 = rr2 - g2 * m;
          const float y8[8] = {oa[0] / L, oa[1] / L, oa[2] / L, oa[3] / L, ob[0] / L, ob[1] / L, ob[2] / L, ob[3] / L};
          store_act8x<false>((u32x4*)outp, cl.row_off + r2, head2 * HD + e0, y8, act_tiles);
        } else {
          float* dst = gpart + ((size_t)(split * T + t) * 16 + mr) * ROW;
          Xwg<true>::st4f(dst + e0, oa);
          Xwg<true>::st4f(dst + e0 + 4, ob);
          if (e0 == 0) Xwg<true>::st4f(dst + HD, f32x4{M, L, 0.f, 0.f});
        }
      }
    }
  }
  if (cl.nsplit == 1) return;

  // ---- count in; the last of the client's splits to arrive merges them ----
  Xwg<true>::drain();  // this thread's partial stores have been acknowledged
  __syncthreads();
  unsigned* counter = counters + cl.count_off + kvh * nz + (int)blockIdx.z;
  if (tid == 0) {
    const unsigned prev = __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int last = prev == (unsigned)cl.nsplit - 1u;
    if (last) __hip_atomic_store(counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // ready for the next launch
    *last_lds = last;
  }
  __syncthreads();
  if (*last_lds == 0) return;
  for (int t = 0; t < T; ++t) {
    const int rr2 = (qt0 + t) * 16 + mr;
    if (qt0 + t >= nqt || mr >= 16 || rr2 >= R) continue;
    const int g2 = div_small(rr2, m_rinv);
    const int head2 = kvh * group + g2, r2 = rr2 - g2 * m;
    float acc[8];
    attn_merge_rows([&](int sp) { return gpart + ((size_t)(sp * T + t) * 16 + mr) * ROW; }, cl.nsplit, HD, e0, acc);
    store_act8x<false>((u32x4*)outp, cl.row_off + r2, head2 * HD + e0, acc, act_tiles);
  }
}

// grid = (threads of the largest client / 64, clients)
__global__ __launch_bounds__(64) void attn_merge_packed_kernel(const float* part, int n_q_heads, int h, AttnBatch batch,
                                                              uint4* outp, int act_tiles, const int32_t* gate) {
  if (gate != nullptr && *gate == 0) return;
  const AttnClient c = batch.c[blockIdx.y];
  attn_merge_thread<false>(part + c.part_off, c.m, n_q_heads, h, c.nsplit, (u32x4*)outp,
                           blockIdx.x * blockDim.x + threadIdx.x, c.row_off, act_tiles);
}

// merge the splits of one (row, head): o = sum_s e^{m_s - M} o_s / sum_s e^{m_s - M} l_s, splits taken
// in index order.  h/8 threads per (row, head), 8 consecutive elements each (fp32 cache path).
__global__ __launch_bounds__(256) void attn_combine_kernel(const float* __restrict__ part, int m, int n_q_heads, int h,
                                                           int nsplit, float* __restrict__ out) {
  const int tpp = h / 8;  // threads per pair
  const int gt = blockIdx.x * blockDim.x + threadIdx.x;
  const int pair = gt / tpp, e0 = (gt % tpp) * 8;  // pair = head * m + r
  if (pair >= m * n_q_heads) return;
  const int head = pair / m, r = pair % m;
  const float* p = part + (size_t)pair * nsplit * (h + kPartPad);
  float M = -INFINITY;
  for (int s = 0; s < nsplit; ++s) M = fmaxf(M, p[(size_t)s * (h + kPartPad) + h]);
  float L = 0.f, acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = 0.f;
  for (int s = 0; s < nsplit; ++s) {
    const float* ps = p + (size_t)s * (h + kPartPad);
    const float ms = ps[h];
    if (ms == -INFINITY) continue;
    const float wgt = expf(ms - M);
    L += ps[h + 1] * wgt;
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] += ps[e0 + i] * wgt;
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] /= L;
#pragma unroll
  for (int i = 0; i < 8; ++i) out[((size_t)r * n_q_heads + head) * h + e0 + i] = acc[i];
}

int attn_nsplit(int total_tokens, int chunk) { return (total_tokens + chunk - 1) / chunk; }

hipError_t launch_attention(const AttnCall& c, hipStream_t st) {
  const int h = c.kv.head_dim;
  const int total = c.start_pos + c.m;
  const int nsplit = attn_nsplit(total, c.chunk);
  if (c.dtype == PIPESD_F32) {
    if (c.chunk > kAttnChunkMax) return hipErrorInvalidValue;
    const size_t lds = (size_t)(2 * kAttnChunkMax * (h + 1) + kMaxRows * h + kMaxRows * kAttnChunkMax) * sizeof(float);
    dim3 grid(c.kv.n_kv_heads, nsplit);
    attn_partial_kernel<float><<<grid, kAttnThreads, lds, st>>>(c.q, c.kv, c.layer, c.m, c.start_pos, c.n_q_heads,
                                                                c.chunk, nsplit, c.part);
  } else {
    const AttnBatch& b = c.batch;
    if (b.n < 1 || b.n > kMaxPassClients) return hipErrorInvalidValue;
    const int group = c.n_q_heads / c.kv.n_kv_heads;
    int splits = 0, max_m = 1;
    long tasks = 0;  // (kv head, split, query tile) over all clients
    for (int i = 0; i < b.n; ++i) {
      splits += b.c[i].nsplit;
      max_m = b.c[i].m > max_m ? b.c[i].m : max_m;
      tasks += (long)c.kv.n_kv_heads * b.c[i].nsplit * ((group * b.c[i].m + 15) / 16);
    }
    if (c.stream_tiles) {  // few rows per client: the streaming kernel (the batch was planned by attn_stream_plan)
      const int T = c.stream_tiles;
      if ((h != 128 && h != 64) || max_m > kStreamMaxRows || (T != 1 && T != 2) || c.counters == nullptr) return hipErrorInvalidValue;
      for (int i = 0; i < b.n; ++i)  // (a lane per step holds the step's block-table entries)
        if (b.c[i].span < kStreamWgTokens || b.c[i].span > kStreamMaxSteps * kStreamWgTokens) return hipErrorInvalidValue;
      const int nz = ((group * max_m + 15) / 16 + T - 1) / T;
      static bool stream_lds_allowed = false;
      if (!stream_lds_allowed) {
        const hipFuncAttribute attr = hipFuncAttributeMaxDynamicSharedMemorySize;
        hipError_t e = hipFuncSetAttribute((const void*)attn_stream_kernel<128, 1>, attr, (int)stream_lds_bytes<128>(1));
        if (e == hipSuccess) e = hipFuncSetAttribute((const void*)attn_stream_kernel<128, 2>, attr, (int)stream_lds_bytes<128>(2));
        if (e == hipSuccess) e = hipFuncSetAttribute((const void*)attn_stream_kernel<64, 1>, attr, (int)stream_lds_bytes<64>(1));
        if (e == hipSuccess) e = hipFuncSetAttribute((const void*)attn_stream_kernel<64, 2>, attr, (int)stream_lds_bytes<64>(2));
        if (e != hipSuccess) return e;
        stream_lds_allowed = true;
      }
      const dim3 grid(c.kv.n_kv_heads, splits, nz), block(kStreamWaves * 64);
      uint4* outp = (uint4*)c.outp;
      if (h == 128 && T == 2)
        attn_stream_kernel<128, 2><<<grid, block, stream_lds_bytes<128>(2), st>>>(c.q, c.kv, c.layer, c.n_q_heads, b, c.part, outp, c.act_tiles, c.gate, c.counters);
      else if (h == 128)
        attn_stream_kernel<128, 1><<<grid, block, stream_lds_bytes<128>(1), st>>>(c.q, c.kv, c.layer, c.n_q_heads, b, c.part, outp, c.act_tiles, c.gate, c.counters);
      else if (T == 2)
        attn_stream_kernel<64, 2><<<grid, block, stream_lds_bytes<64>(2), st>>>(c.q, c.kv, c.layer, c.n_q_heads, b, c.part, outp, c.act_tiles, c.gate, c.counters);
      else
        attn_stream_kernel<64, 1><<<grid, block, stream_lds_bytes<64>(1), st>>>(c.q, c.kv, c.layer, c.n_q_heads, b, c.part, outp, c.act_tiles, c.gate, c.counters);
      return hipGetLastError();
    }
    // more tasks than the device holds at once (two workgroups per compute unit): a workgroup walks
    // several query tiles with its keys and values in registers, as many as still leave about two
    // workgroups per compute unit (a 128-row prompt block has 32 tiles per (kv head, split))
    const int max_qt = (group * max_m + 15) / 16, n_cu = device_cu_count();
    const int qpw = tasks > 4L * n_cu ? (int)std::max(1L, std::min((long)max_qt, tasks / (2L * n_cu))) : 1;
    dim3 grid(c.kv.n_kv_heads, splits, (max_qt + qpw - 1) / qpw);
    if (h != 128 && h != 64) return hipErrorInvalidValue;
    const size_t lds = attn_lds_floats(h) * sizeof(float);
    static bool lds_allowed = false;  // more than 64 KB of dynamic LDS has to be asked for once per kernel
    if (!lds_allowed) {
      const int b128 = (int)(attn_lds_floats(128) * sizeof(float)), b64 = (int)(attn_lds_floats(64) * sizeof(float));
      const hipFuncAttribute attr = hipFuncAttributeMaxDynamicSharedMemorySize;
      hipError_t e = hipFuncSetAttribute((const void*)attn_mfma_kernel<128, false>, attr, b128);
      if (e == hipSuccess) e = hipFuncSetAttribute((const void*)attn_mfma_kernel<128, true>, attr, b128);
      if (e == hipSuccess) e = hipFuncSetAttribute((const void*)attn_mfma_kernel<64, false>, attr, b64);
      if (e == hipSuccess) e = hipFuncSetAttribute((const void*)attn_mfma_kernel<64, true>, attr, b64);
      if (e != hipSuccess) return e;
      lds_allowed = true;
    }
    const dim3 block(kAttnWaves * 64);
    if (h == 128 && qpw > 1)
      attn_mfma_kernel<128, true><<<grid, block, lds, st>>>(c.q, c.kv, c.layer, c.n_q_heads, b, c.part, qpw, c.gate);
    else if (h == 128)
      attn_mfma_kernel<128, false><<<grid, block, lds, st>>>(c.q, c.kv, c.layer, c.n_q_heads, b, c.part, qpw, c.gate);
    else if (qpw > 1)
      attn_mfma_kernel<64, true><<<grid, block, lds, st>>>(c.q, c.kv, c.layer, c.n_q_heads, b, c.part, qpw, c.gate);
    else
      attn_mfma_kernel<64, false><<<grid, block, lds, st>>>(c.q, c.kv, c.layer, c.n_q_heads, b, c.part, qpw, c.gate);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (c.dtype == PIPESD_F32) {
    const int threads = c.m * c.n_q_heads * (h / 8);
    attn_combine_kernel<<<(threads + 255) / 256, 256, 0, st>>>(c.part, c.m, c.n_q_heads, h, nsplit, c.out);
  } else {
    int max_m = 1;
    for (int i = 0; i < c.batch.n; ++i) max_m = c.batch.c[i].m > max_m ? c.batch.c[i].m : max_m;
    const int threads = max_m * c.n_q_heads * (h / 8);
    attn_merge_packed_kernel<<<dim3((threads + 63) / 64, c.batch.n), 64, 0, st>>>(c.part, c.n_q_heads, h, c.batch,
                                                                                   (uint4*)c.outp, c.act_tiles, c.gate);
  }
  return hipGetLastError();
}

int attn_chunk_tokens(int dtype) { return dtype == PIPESD_F32 ? kAttnChunkMax : kAttnWgTokens; }
int attn_stream_plan(int n_q_heads, int n_kv_heads, int head_dim, AttnBatch& b, size_t* part_floats) {
  *part_floats = 0;
  if (b.n < 1 || b.n > kMaxPassClients || (head_dim != 128 && head_dim != 64)) return 0;
  const int group = n_q_heads / n_kv_heads;
  int max_m = 1;
  long tasks = 0;  // (kv head, split, query tile) over all clients
  for (int i = 0; i < b.n; ++i) {
    AttnClient& cl = b.c[i];
    if (cl.m > kStreamMaxRows || (cl.m > kMaxRows && b.n != 1)) return 0;
    max_m = std::max(max_m, (int)cl.m);
    const int total = cl.start_pos + cl.m;
    cl.span = kStreamMinSpan;
    if (cl.m <= kMaxRows) {
      while ((total + cl.span - 1) / cl.span > kStreamMaxSplits) cl.span *= 2;
    } else {
      // a prompt block (alone in its pass): the query tiles alone give many workgroups, so the context
      // is cut only as far as it takes to have about two workgroups per compute unit
      const long groups = (long)n_kv_heads * (((group * cl.m + 15) / 16 + 1) / 2);
      const long fit = ((long)total + kStreamMaxSteps * kStreamWgTokens - 1) / (kStreamMaxSteps * kStreamWgTokens);
      const long want = std::max(fit, std::min((long)kStreamMaxSplits, 2L * device_cu_count() / groups));
      const int steps = (total + kStreamMinSpan - 1) / kStreamMinSpan;
      cl.span = (int)((steps + want - 1) / want) * kStreamMinSpan;
    }
    cl.nsplit = (total + cl.span - 1) / cl.span;
    if (cl.span > kStreamMaxSteps * kStreamWgTokens || cl.nsplit > kStreamMaxSplits) return 0;  // (contexts beyond 131072 tokens)
    tasks += (long)n_kv_heads * cl.nsplit * ((group * cl.m + 15) / 16);
  }
  // two tiles per workgroup (keys and values read once for both) where a head group has exactly
  // two, or where single tiles would be more workgroups than two rounds of the device
  const int max_qt = (group * max_m + 15) / 16;
  const int T = (max_qt == 2 || tasks > 2L * device_cu_count()) ? 2 : 1;
  const int nz = (max_qt + T - 1) / T;
  if ((long)n_kv_heads * nz > kAttnCounters / kMaxPassClients) return 0;
  size_t floats = 0;
  for (int i = 0; i < b.n; ++i) {
    AttnClient& cl = b.c[i];
    if (floats > (size_t)INT32_MAX) return 0;
    cl.part_off = (int32_t)floats;
    cl.count_off = i * (kAttnCounters / kMaxPassClients);
    floats += (size_t)n_kv_heads * nz * cl.nsplit * T * 16 * (head_dim + kPartPad);
  }
  *part_floats = floats;
  return T;
}

}  // namespace pipesd
