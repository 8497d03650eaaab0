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

// merge the splits of one (row, head): o = sum_s e^{m_s - M} o_s / sum_s e^{m_s - M} l_s
__global__ void attn_combine_kernel(const float* __restrict__ part, int m, int n_q_heads, int h, int nsplit,
                                    float* __restrict__ out) {
  const int r = blockIdx.x, head = blockIdx.y;
  const float* p = part + ((size_t)head * m + r) * nsplit * (h + 2);
  float M = -INFINITY;
  for (int s = 0; s < nsplit; ++s) M = fmaxf(M, p[(size_t)s * (h + 2) + h]);
  float L = 0.f;
  for (int s = 0; s < nsplit; ++s) {
    const float ms = p[(size_t)s * (h + 2) + h];
    if (ms != -INFINITY) L += p[(size_t)s * (h + 2) + h + 1] * expf(ms - M);
  }
  for (int e = threadIdx.x; e < h; e += blockDim.x) {
    float acc = 0.f;
    for (int s = 0; s < nsplit; ++s) {
      const float ms = p[(size_t)s * (h + 2) + h];
      if (ms != -INFINITY) acc += p[(size_t)s * (h + 2) + e] * expf(ms - M);
    }
    out[((size_t)r * n_q_heads + head) * h + e] = acc / L;
  }
}

int attn_nsplit(int total_tokens, int chunk) { return (total_tokens + chunk - 1) / chunk; }

hipError_t launch_attention(const AttnCall& c, hipStream_t st) {
  const int h = c.kv.head_dim;
  const int total = c.start_pos + c.m;
  const int nsplit = attn_nsplit(total, c.chunk);
  if (c.chunk > kAttnChunkMax) return hipErrorInvalidValue;
  const size_t lds = (size_t)(2 * kAttnChunkMax * (h + 1) + kMaxRows * h + kMaxRows * kAttnChunkMax) * sizeof(float);
  dim3 grid(c.kv.n_kv_heads, nsplit);
  if (c.dtype == PIPESD_F32)
    attn_partial_kernel<float><<<grid, kAttnThreads, lds, st>>>(c.q, c.kv, c.layer, c.m, c.start_pos, c.n_q_heads,
                                                                c.chunk, nsplit, c.part);
  else
    attn_partial_kernel<uint16_t><<<grid, kAttnThreads, lds, st>>>(c.q, c.kv, c.layer, c.m, c.start_pos, c.n_q_heads,
                                                                   c.chunk, nsplit, c.part);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  dim3 g2(c.m, c.n_q_heads);
  attn_combine_kernel<<<g2, 128, 0, st>>>(c.part, c.m, c.n_q_heads, h, nsplit, c.out);
  return hipGetLastError();
}

}  // namespace pipesd
