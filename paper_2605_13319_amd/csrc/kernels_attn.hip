// Grouped-query attention of the m = k + 1 causal rows of a pass over the paged KV cache.
// (Masked self-attention of a decoder-only layer, Sec. 2.1; row r sees key positions 0..pos_r.)
//
// Split over the context: workgroup (kv_head, split) handles `chunk` consecutive tokens for every
// query row of the query heads that share the KV head, producing an un-normalised partial
// (max, sum, o); a second kernel merges the splits in a fixed order, so results do not depend on
// scheduling.
#include <algorithm>

#include "device_attn.h"

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

}  // namespace pipesd
