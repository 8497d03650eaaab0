// Grouped-query attention of the m = k + 1 causal rows of a pass over the paged KV cache.
// (Masked self-attention of a decoder-only layer, Sec. 2.1; row r sees key positions 0..pos_r.)
//
// Split over the context: workgroup (kv_head, split) handles `chunk` consecutive tokens for every
// query row of the query heads that share the KV head, producing an un-normalised partial
// (max, sum, o); a second kernel merges the splits in a fixed order, so results do not depend on
// scheduling.
#include "common.h"

namespace pipesd {

constexpr int kAttnThreads = 256;
constexpr int kPartPad = 4;  // a partial row is [head_dim values, max, sum, 2 unused] so that rows stay 16-byte aligned
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
// bf16 cache: the same computation on the matrix cores.
//
// A wave loads 32 tokens' keys (two [16 tok][h] blocks, A operand of S^T = K Q^T) and values (two
// [h][16 tok] blocks, A operand of O^T = V^T P) straight from the paged cache in MFMA operand
// layout.  Queries and probabilities are fed as bf16 hi + lo pairs so only the cache itself is
// bf16.  The scores of one query row sit in the four lanes {c, c+16, c+32, c+48}, so the softmax
// statistics take two cross-lane steps.
// ------------------------------------------------------------------------------------------------
typedef __attribute__((ext_vector_type(4))) unsigned au32x4;
typedef __attribute__((ext_vector_type(2))) unsigned au32x2;

__device__ __forceinline__ void split_hi_lo8(const float (&v)[8], bf16x8& hi, bf16x8& lo) {
  unsigned h[4], l[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint16_t h0 = f32_to_bf16_bits(v[2 * i]), h1 = f32_to_bf16_bits(v[2 * i + 1]);
    const uint16_t l0 = f32_to_bf16_bits(v[2 * i] - bf16_bits_to_f32(h0));
    const uint16_t l1 = f32_to_bf16_bits(v[2 * i + 1] - bf16_bits_to_f32(h1));
    h[i] = (unsigned)h0 | ((unsigned)h1 << 16);
    l[i] = (unsigned)l0 | ((unsigned)l1 << 16);
  }
  hi = __builtin_bit_cast(bf16x8, au32x4{h[0], h[1], h[2], h[3]});
  lo = __builtin_bit_cast(bf16x8, au32x4{l[0], l[1], l[2], l[3]});
}

constexpr int kAttnWaves = 8;
constexpr int kAttnWgTokens = kAttnWaves * 32;

// Workgroup (kv_head, split) = 8 waves x 32 tokens.  A wave loads its 32 tokens' keys and values once
// into registers, then walks the 16-row tiles of the query rows that share the KV head; per tile
// the eight waves' (max, sum, O) are merged pairwise through LDS and written as the split's
// partial; a second small kernel merges the splits.
template <int HD>
__global__ __launch_bounds__(kAttnWaves * 64) void attn_mfma_kernel(const float* __restrict__ q, KvView kv, int layer,
                                                                    int m, int start_pos, int n_q_heads, int nsplit,
                                                                    float* __restrict__ part) {
  constexpr int KSQ = HD / 32, HT = HD / 16, ROW = HD + 4;
  __shared__ float o_lds[kAttnWaves / 2][16][ROW];
  __shared__ float m_lds[kAttnWaves / 2][16], l_lds[kAttnWaves / 2][16];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int c = lane & 15, g = lane >> 4;
  const int kvh = blockIdx.x, split = blockIdx.y;
  const int group = n_q_heads / kv.n_kv_heads;
  const int R = group * m, NQ = (R + 15) / 16;
  const int total = start_pos + m;
  const int tok0 = split * kAttnWgTokens + w * 32;
  const uint16_t* pool = (const uint16_t*)kv.pool;
  const float scale = 1.0f / sqrtf((float)HD);

  // keys and values of this wave's 32 tokens; tokens at or beyond `total` read as zero
  bf16x8 kf[2][KSQ], vf[HT];
  {
    au32x2 vlo[HT], vhi[HT];
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
      const int tb = tok0 + tt * 16;
      const int blk = tb < total ? kv.table[tb / kBlockTokens] : 0;
      const int64_t base = (int64_t)layer * kv.layer_stride + (int64_t)blk * kv.block_elems;
      const bool tok_ok = tb + c < total;
#pragma unroll
      for (int s = 0; s < KSQ; ++s) {
        au32x4 v = au32x4{0u, 0u, 0u, 0u};
        if (tok_ok) v = *(const au32x4*)(pool + base + ((int64_t)kvh * kBlockTokens + c) * HD + s * 32 + g * 8);
        kf[tt][s] = __builtin_bit_cast(bf16x8, v);
      }
      const int nvalid = min(4, max(0, total - (tb + g * 4)));
      const unsigned long long keep = nvalid >= 4 ? ~0ull : ((1ull << (16 * nvalid)) - 1ull);
#pragma unroll
      for (int j = 0; j < HT; ++j) {
        au32x2 v = au32x2{0u, 0u};
        if (nvalid > 0)
          v = *(const au32x2*)(pool + base + kv.v_offset + ((int64_t)kvh * HD + j * 16 + c) * kBlockTokens + g * 4);
        v.x &= (unsigned)keep;
        v.y &= (unsigned)(keep >> 32);
        if (tt == 0) vlo[j] = v; else vhi[j] = v;
      }
    }
#pragma unroll
    for (int j = 0; j < HT; ++j)
      vf[j] = __builtin_bit_cast(bf16x8, au32x4{vlo[j].x, vlo[j].y, vhi[j].x, vhi[j].y});
  }

  for (int qt = 0; qt < NQ; ++qt) {
    const int rr = qt * 16 + c;
    const bool row_ok = rr < R;
    const int gq = row_ok ? rr / m : 0, r = row_ok ? rr % m : 0;
    const int head = kvh * group + gq;
    bf16x8 qhi[KSQ], qlo[KSQ];
#pragma unroll
    for (int s = 0; s < KSQ; ++s) {
      float v[8];
      if (row_ok) {
        const float* qp = q + ((size_t)r * n_q_heads + head) * HD + s * 32 + g * 8;
        const float4 x0 = *(const float4*)qp, x1 = *(const float4*)(qp + 4);
        v[0] = x0.x; v[1] = x0.y; v[2] = x0.z; v[3] = x0.w;
        v[4] = x1.x; v[5] = x1.y; v[6] = x1.z; v[7] = x1.w;
      } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = 0.f;
      }
      split_hi_lo8(v, qhi[s], qlo[s]);
    }
    // scores of query row c against tokens tok0 + tt*16 + g*4 + i
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
      for (int i = 0; i < 4; ++i) {
        const int t = tok0 + tt * 16 + g * 4 + i;
        sc[tt * 4 + i] = (row_ok && t <= pos_q) ? acc[i] * scale : -INFINITY;
      }
    }
    float m_run = sc[0];
#pragma unroll
    for (int i = 1; i < 8; ++i) m_run = fmaxf(m_run, sc[i]);
    m_run = fmaxf(m_run, __shfl_xor(m_run, 16, 64));
    m_run = fmaxf(m_run, __shfl_xor(m_run, 32, 64));
    float pv[8], l_run = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      pv[i] = (sc[i] == -INFINITY) ? 0.f : expf(sc[i] - m_run);
      l_run += pv[i];
    }
    l_run += __shfl_xor(l_run, 16, 64);
    l_run += __shfl_xor(l_run, 32, 64);
    bf16x8 phi, plo;
    split_hi_lo8(pv, phi, plo);
    f32x4 o[HT];
#pragma unroll
    for (int j = 0; j < HT; ++j) {
      f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[j], phi, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[j], plo, acc, 0, 0, 0);
      o[j] = acc;  // O[query c][element j*16 + g*4 + i]
    }
    // merge the eight waves pairwise through LDS: (4..7 -> 0..3), (2,3 -> 0,1), (1 -> 0)
#pragma unroll
    for (int span = kAttnWaves / 2; span >= 1; span >>= 1) {
      if (w >= span && w < 2 * span) {
#pragma unroll
        for (int j = 0; j < HT; ++j) *(f32x4*)&o_lds[w - span][c][j * 16 + g * 4] = o[j];
        if (g == 0) {
          m_lds[w - span][c] = m_run;
          l_lds[w - span][c] = l_run;
        }
      }
      __syncthreads();
      if (w < span) {
        const float mp = m_lds[w][c], lp = l_lds[w][c];
        const float nm = fmaxf(m_run, mp);
        const float so = (m_run == -INFINITY) ? 0.f : expf(m_run - nm);
        const float sp = (mp == -INFINITY) ? 0.f : expf(mp - nm);
        l_run = l_run * so + lp * sp;
        m_run = nm;
#pragma unroll
        for (int j = 0; j < HT; ++j) {
          const f32x4 op = *(const f32x4*)&o_lds[w][c][j * 16 + g * 4];
          o[j] = o[j] * so + op * sp;
        }
      }
      __syncthreads();
    }
    if (w == 0 && row_ok) {
      float* dst = part + (((size_t)head * m + r) * nsplit + split) * (HD + kPartPad);
#pragma unroll
      for (int j = 0; j < HT; ++j) *(f32x4*)(dst + j * 16 + g * 4) = o[j];
      if (g == 0) *(f32x4*)(dst + HD) = f32x4{m_run, l_run, 0.f, 0.f};
    }
  }
}


// Merge the splits of one (row, head) for the bf16 path: one thread per 8 consecutive elements, all
// of a batch's loads issued before any is used; the result is written packed for the O projection.
__global__ __launch_bounds__(64) void attn_merge_packed_kernel(const float* __restrict__ part, int m, int n_q_heads,
                                                              int h, int nsplit, uint4* outp) {
  constexpr int BATCH = 9;
  const int segs = h / 8;
  const int gt = blockIdx.x * blockDim.x + threadIdx.x;
  const int pair = gt / segs, e0 = (gt % segs) * 8;  // pair = head * m + r
  if (pair >= m * n_q_heads) return;
  const int head = pair / m, r = pair % m;
  const float* p = part + (size_t)pair * nsplit * (h + kPartPad);
  float M = -INFINITY, L = 0.f, acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = 0.f;
  for (int s0 = 0; s0 < nsplit; s0 += BATCH) {
    f32x4 ml[BATCH], oa[BATCH], ob[BATCH];
#pragma unroll
    for (int j = 0; j < BATCH; ++j) {
      const float* ps = p + (size_t)min(s0 + j, nsplit - 1) * (h + kPartPad);
      ml[j] = *(const f32x4*)(ps + h);
      oa[j] = *(const f32x4*)(ps + e0);
      ob[j] = *(const f32x4*)(ps + e0 + 4);
    }
    float bm = M;
#pragma unroll
    for (int j = 0; j < BATCH; ++j)
      if (s0 + j < nsplit) bm = fmaxf(bm, ml[j][0]);
    if (bm == -INFINITY) continue;
    const float so = (M == -INFINITY) ? 0.f : expf(M - bm);
    L *= so;
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] *= so;
#pragma unroll
    for (int j = 0; j < BATCH; ++j) {
      const float wgt = (s0 + j < nsplit && ml[j][0] != -INFINITY) ? expf(ml[j][0] - bm) : 0.f;
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
  store_act8(outp, r, head * h + e0, acc);
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
    const int nsp = attn_nsplit(total, kAttnWgTokens);
    dim3 grid(c.kv.n_kv_heads, nsp);
    if (h == 128)
      attn_mfma_kernel<128><<<grid, kAttnWaves * 64, 0, st>>>(c.q, c.kv, c.layer, c.m, c.start_pos, c.n_q_heads, nsp,
                                                              c.part);
    else if (h == 64)
      attn_mfma_kernel<64><<<grid, kAttnWaves * 64, 0, st>>>(c.q, c.kv, c.layer, c.m, c.start_pos, c.n_q_heads, nsp,
                                                             c.part);
    else
      return hipErrorInvalidValue;
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int threads = c.m * c.n_q_heads * (h / 8);
  if (c.dtype == PIPESD_F32)
    attn_combine_kernel<<<(threads + 255) / 256, 256, 0, st>>>(c.part, c.m, c.n_q_heads, h, nsplit, c.out);
  else
    attn_merge_packed_kernel<<<(threads + 63) / 64, 64, 0, st>>>(c.part, c.m, c.n_q_heads, h,
                                                                 attn_nsplit(total, kAttnWgTokens), (uint4*)c.outp);
  return hipGetLastError();
}

int attn_chunk_tokens(int dtype) { return dtype == PIPESD_F32 ? kAttnChunkMax : kAttnWgTokens; }

}  // namespace pipesd
