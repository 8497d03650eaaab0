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
      float* o = part + (((size_t)head * m + tid) * nsplit + split) * (h + 2);
      o[h] = mx;
      o[h + 1] = l;
    }
    __syncthreads();
    // o = P V
    for (int i = tid; i < m * h; i += kAttnThreads) {
      const int r = i / h, e = i % h;
      float acc = 0.f;
      for (int t = 0; t < nt; ++t) acc = fmaf(ps[r * chunk + t], vs[t * hp + e], acc);
      part[(((size_t)head * m + r) * nsplit + split) * (h + 2) + e] = acc;
    }
  }
}

// ------------------------------------------------------------------------------------------------
// bf16 cache: the same computation on the matrix cores.
//
// Workgroup (kv_head, split) = 4 waves x 32 tokens.  A wave loads its 32 tokens' keys (two
// [16 tok][h] blocks, A operand of S^T = K Q^T) and values (two [h][16 tok] blocks, A operand of
// O^T = V^T P) once into registers, straight from the paged cache in MFMA operand layout, then
// walks the 16-row tiles of the query rows that share the KV head.  Queries and probabilities are
// fed as bf16 hi + lo pairs so only the cache itself is bf16.  The scores of one query row sit in
// the four lanes {c, c+16, c+32, c+48}, so the softmax statistics take two cross-lane steps.
// The four waves' (max, sum, O) are merged through LDS and written as one partial per split.
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

constexpr int kAttnWaves = 4;
constexpr int kAttnWgTokens = kAttnWaves * 32;

template <int HD>
__global__ __launch_bounds__(kAttnWaves * 64) void attn_mfma_kernel(const float* __restrict__ q, KvView kv, int layer,
                                                                    int m, int start_pos, int n_q_heads, int nsplit,
                                                                    float* __restrict__ part) {
  constexpr int KSQ = HD / 32, HT = HD / 16, ROW = HD + 4;
  __shared__ float o_lds[kAttnWaves][16][ROW];
  __shared__ float m_lds[kAttnWaves][16], l_lds[kAttnWaves][16];
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
      const bool blk_ok = tb < total;
      const int blk = blk_ok ? kv.table[tb / kBlockTokens] : 0;
      const int64_t base = (int64_t)layer * kv.layer_stride + (int64_t)blk * kv.block_elems;
      const bool tok_ok = tb + c < total;
#pragma unroll
      for (int s = 0; s < KSQ; ++s) {
        au32x4 v = au32x4{0u, 0u, 0u, 0u};
        if (tok_ok) v = *(const au32x4*)(pool + base + ((int64_t)kvh * kBlockTokens + c) * HD + s * 32 + g * 8);
        kf[tt][s] = __builtin_bit_cast(bf16x8, v);
      }
      // values: element row e = j*16 + c, tokens g*4 .. g*4+3 of this block
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
    float mx = sc[0];
#pragma unroll
    for (int i = 1; i < 8; ++i) mx = fmaxf(mx, sc[i]);
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    float pv[8], l = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      pv[i] = (sc[i] == -INFINITY) ? 0.f : expf(sc[i] - mx);
      l += pv[i];
    }
    l += __shfl_xor(l, 16, 64);
    l += __shfl_xor(l, 32, 64);
    bf16x8 phi, plo;
    split_hi_lo8(pv, phi, plo);
#pragma unroll
    for (int j = 0; j < HT; ++j) {
      f32x4 o = f32x4{0.f, 0.f, 0.f, 0.f};
      o = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[j], phi, o, 0, 0, 0);
      o = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[j], plo, o, 0, 0, 0);
      *(f32x4*)&o_lds[w][c][j * 16 + g * 4] = o;  // O[query c][element j*16 + g*4 + i]
    }
    if (g == 0) {
      m_lds[w][c] = mx;
      l_lds[w][c] = l;
    }
    __syncthreads();
    // merge the four waves and write the split's partial
    {
      const int cc = tid >> 4, seg = tid & 15;
      const int row = qt * 16 + cc;
      if (row < R) {
        float M = m_lds[0][cc];
#pragma unroll
        for (int ww = 1; ww < kAttnWaves; ++ww) M = fmaxf(M, m_lds[ww][cc]);
        float wgt[kAttnWaves], L = 0.f;
#pragma unroll
        for (int ww = 0; ww < kAttnWaves; ++ww) {
          const float mw = m_lds[ww][cc];
          wgt[ww] = (mw == -INFINITY) ? 0.f : expf(mw - M);
          L += l_lds[ww][cc] * wgt[ww];
        }
        const int hq = kvh * group + row / m, rq = row % m;
        float* dst = part + (((size_t)hq * m + rq) * nsplit + split) * (HD + 2);
#pragma unroll
        for (int x = 0; x < HD / 16; ++x) {
          const int e = seg * (HD / 16) + x;
          float acc = 0.f;
#pragma unroll
          for (int ww = 0; ww < kAttnWaves; ++ww) acc += o_lds[ww][cc][e] * wgt[ww];
          dst[e] = acc;
        }
        if (seg == 0) {
          dst[HD] = M;
          dst[HD + 1] = L;
        }
      }
    }
    __syncthreads();
  }
}

// merge the splits of one (row, head): o = sum_s e^{m_s - M} o_s / sum_s e^{m_s - M} l_s, splits taken
// in index order.  h/8 threads per (row, head), 8 consecutive elements each; the result goes out as
// fp32 or, for the next GEMM, packed (ActPack).
template <bool PACKED>
__global__ __launch_bounds__(256) void attn_combine_kernel(const float* __restrict__ part, int m, int n_q_heads, int h,
                                                           int nsplit, float* __restrict__ out, uint4* outp) {
  const int tpp = h / 8;  // threads per pair
  const int gt = blockIdx.x * blockDim.x + threadIdx.x;
  const int pair = gt / tpp, e0 = (gt % tpp) * 8;  // pair = head * m + r
  if (pair >= m * n_q_heads) return;
  const int head = pair / m, r = pair % m;
  const float* p = part + (size_t)pair * nsplit * (h + 2);
  float M = -INFINITY;
  for (int s = 0; s < nsplit; ++s) M = fmaxf(M, p[(size_t)s * (h + 2) + h]);
  float L = 0.f, acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = 0.f;
  for (int s = 0; s < nsplit; ++s) {
    const float* ps = p + (size_t)s * (h + 2);
    const float ms = ps[h];
    if (ms == -INFINITY) continue;
    const float wgt = expf(ms - M);
    L += ps[h + 1] * wgt;
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] += ps[e0 + i] * wgt;
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] /= L;
  if (PACKED) {
    store_act8(outp, r, head * h + e0, acc);
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i) out[((size_t)r * n_q_heads + head) * h + e0 + i] = acc[i];
  }
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
    if (c.chunk != kAttnWgTokens) return hipErrorInvalidValue;
    dim3 grid(c.kv.n_kv_heads, nsplit);
    if (h == 128)
      attn_mfma_kernel<128><<<grid, kAttnWaves * 64, 0, st>>>(c.q, c.kv, c.layer, c.m, c.start_pos, c.n_q_heads, nsplit,
                                                              c.part);
    else if (h == 64)
      attn_mfma_kernel<64><<<grid, kAttnWaves * 64, 0, st>>>(c.q, c.kv, c.layer, c.m, c.start_pos, c.n_q_heads, nsplit,
                                                             c.part);
    else
      return hipErrorInvalidValue;
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int threads = c.m * c.n_q_heads * (h / 8);
  if (c.dtype == PIPESD_F32)
    attn_combine_kernel<false><<<(threads + 255) / 256, 256, 0, st>>>(c.part, c.m, c.n_q_heads, h, nsplit, c.out,
                                                                      nullptr);
  else
    attn_combine_kernel<true><<<(threads + 255) / 256, 256, 0, st>>>(c.part, c.m, c.n_q_heads, h, nsplit, nullptr,
                                                                     (uint4*)c.outp);
  return hipGetLastError();
}

int attn_chunk_tokens(int dtype) { return dtype == PIPESD_F32 ? kAttnChunkMax : kAttnWgTokens; }

}  // namespace pipesd
