// Row setup, the plain-ALU fp32 layer kernels, and KV bookkeeping kernels.
#include "common.h"

namespace pipesd {

// ---------------------------------------------------------------------------------------------
// Row setup: x_r = E[token_r] (fp32 residual stream) and cos/sin(pos_r * theta_i), the angle
// evaluated in fp64 and rounded once (rotary positions; the target forward of Sec. 2.2).
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ void setup_rows_kernel(const T* __restrict__ emb, PassTokens toks, RowMap map, int m, int d, int half,
                                  const double* __restrict__ theta, float* __restrict__ xres,
                                  float* __restrict__ rope_cs, const float* __restrict__ gain, uint4* xpk,
                                  int act_tiles, float* __restrict__ ssq_out, int ssq_stride,
                                  RowMap* __restrict__ map_dev) {
  __shared__ float red[4];
  const int r = blockIdx.x;
  if (r >= m) return;
  if (map_dev != nullptr && r == 0 && threadIdx.x < kMaxPassRows) {
    map_dev->pos[threadIdx.x] = map.pos[threadIdx.x];
    map_dev->table_off[threadIdx.x] = map.table_off[threadIdx.x];
  }
  const size_t base = (size_t)toks.tok[r] * d;
  float sq = 0.f;
  for (int j = threadIdx.x; j < d / 8; j += blockDim.x) {
    float v[8], y[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      v[i] = load_elem(emb, base + j * 8 + i);
      xres[(size_t)r * d + j * 8 + i] = v[i];
      sq = fmaf(v[i], v[i], sq);
    }
    if (xpk != nullptr) {
#pragma unroll
      for (int i = 0; i < 8; ++i) y[i] = v[i] * gain[j * 8 + i];
      store_act8(xpk, r, j * 8, y, act_tiles);
    }
  }
  for (int i = (d / 8) * 8 + threadIdx.x; i < d; i += blockDim.x) xres[(size_t)r * d + i] = load_elem(emb, base + i);
  if (ssq_out != nullptr) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) sq += __shfl_xor(sq, o, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = sq;
    __syncthreads();
    if (threadIdx.x == 0) ssq_out[(size_t)r * ssq_stride] = (red[0] + red[1]) + (red[2] + red[3]);
  }
  for (int i = threadIdx.x; i < half; i += blockDim.x) {
    const double ang = (double)map.pos[r] * theta[i];
    rope_cs[((size_t)r * half + i) * 2 + 0] = (float)cos(ang);
    rope_cs[((size_t)r * half + i) * 2 + 1] = (float)sin(ang);
  }
}

hipError_t launch_setup_rows(int dtype, const void* tok_emb, const PassTokens& toks, const RowMap& map, int m,
                             int d_model, int head_dim, const double* theta, float* xres, float* rope_cs,
                             const float* gain, void* xpk, int act_tiles, float* ssq_out, int ssq_stride,
                             RowMap* map_dev, hipStream_t st) {
  if (dtype == PIPESD_F32)
    setup_rows_kernel<float><<<m, 256, 0, st>>>((const float*)tok_emb, toks, map, m, d_model, head_dim / 2, theta, xres,
                                                rope_cs, nullptr, nullptr, 0, nullptr, 0, map_dev);
  else
    setup_rows_kernel<uint16_t><<<m, 256, 0, st>>>((const uint16_t*)tok_emb, toks, map, m, d_model, head_dim / 2, theta,
                                                   xres, rope_cs, gain, (uint4*)xpk, act_tiles, ssq_out, ssq_stride,
                                                   map_dev);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// fp32 path
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// h = x * rsqrt(mean(x^2) + eps) * g, one workgroup per row
__global__ void rmsnorm_rows_kernel(const float* __restrict__ x, const float* __restrict__ g, float eps, int d,
                                    float* __restrict__ out) {
  __shared__ float red[4];
  const int r = blockIdx.x;
  float s = 0.f;
  for (int i = threadIdx.x; i < d; i += blockDim.x) {
    const float v = x[(size_t)r * d + i];
    s += v * v;
  }
  s = wave_sum(s);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
  __syncthreads();
  const float tot = red[0] + red[1] + red[2] + red[3];
  const float rstd = 1.0f / sqrtf(tot / (float)d + eps);
  for (int i = threadIdx.x; i < d; i += blockDim.x) out[(size_t)r * d + i] = x[(size_t)r * d + i] * rstd * g[i];
}

hipError_t launch_rmsnorm_rows(const float* x, const float* gain, float eps, int m, int d, float* out, hipStream_t st) {
  rmsnorm_rows_kernel<<<m, 256, 0, st>>>(x, gain, eps, d, out);
  return hipGetLastError();
}

// out[r][n] (+)= sum_k act[r][k] * w[n][k]; one wave per output column, lanes stride over K
__global__ void gemm_f32_kernel(const float* __restrict__ act, int lda, const float* __restrict__ w, int N, int K, int m,
                                float* __restrict__ out, int ldo, int add_to_out) {
  const int lane = threadIdx.x & 63;
  const int n = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (n >= N) return;
  float acc[kMaxRows];
#pragma unroll
  for (int r = 0; r < kMaxRows; ++r) acc[r] = 0.f;
  for (int k = lane; k < K; k += 64) {
    const float wv = w[(size_t)n * K + k];
#pragma unroll
    for (int r = 0; r < kMaxRows; ++r)
      if (r < m) acc[r] = fmaf(act[(size_t)r * lda + k], wv, acc[r]);
  }
#pragma unroll
  for (int r = 0; r < kMaxRows; ++r) {
    if (r < m) {
      const float v = wave_sum(acc[r]);
      if (lane == 0) {
        float* o = out + (size_t)r * ldo + n;
        *o = add_to_out ? (*o + v) : v;
      }
    }
  }
}

hipError_t launch_gemm_f32(const float* act, int lda, const float* w, int N, int K, int m, float* out, int ldo,
                           int add_to_out, hipStream_t st) {
  const int waves = 4;
  gemm_f32_kernel<<<(N + waves - 1) / waves, waves * 64, 0, st>>>(act, lda, w, N, K, m, out, ldo, add_to_out);
  return hipGetLastError();
}

// rotate q and k, store q to the query buffer and k, v to the paged cache (fp32 cache)
__global__ void rope_append_f32_kernel(const float* __restrict__ qkv, int m, int start_pos, int layer, int n_q_heads,
                                       KvView kv, const float* __restrict__ rope_cs, float* __restrict__ qbuf) {
  const int h = kv.head_dim, half = h / 2;
  const int n_heads = n_q_heads + 2 * kv.n_kv_heads;
  const int ld = n_heads * h;
  const int r = blockIdx.y, hd = blockIdx.x;
  float* kvp = (float*)kv.pool;
  for (int i = threadIdx.x; i < half; i += blockDim.x) {
    const float a = qkv[(size_t)r * ld + hd * h + i], b = qkv[(size_t)r * ld + hd * h + i + half];
    const float c = rope_cs[((size_t)r * half + i) * 2], s = rope_cs[((size_t)r * half + i) * 2 + 1];
    if (hd < n_q_heads) {
      qbuf[(size_t)r * n_q_heads * h + hd * h + i] = a * c - b * s;
      qbuf[(size_t)r * n_q_heads * h + hd * h + i + half] = b * c + a * s;
    } else if (hd < n_q_heads + kv.n_kv_heads) {
      const int kvh = hd - n_q_heads;
      kvp[k_index(kv, layer, start_pos + r, kvh, i)] = a * c - b * s;
      kvp[k_index(kv, layer, start_pos + r, kvh, i + half)] = b * c + a * s;
    } else {
      const int kvh = hd - n_q_heads - kv.n_kv_heads;
      kvp[v_index(kv, layer, start_pos + r, kvh, i)] = a;
      kvp[v_index(kv, layer, start_pos + r, kvh, i + half)] = b;
    }
  }
}

hipError_t launch_rope_append_f32(const float* qkv, int m, int start_pos, int layer, int n_q_heads, const KvView& kv,
                                  const float* rope_cs, float* qbuf, hipStream_t st) {
  dim3 grid(n_q_heads + 2 * kv.n_kv_heads, m);
  rope_append_f32_kernel<<<grid, 64, 0, st>>>(qkv, m, start_pos, layer, n_q_heads, kv, rope_cs, qbuf);
  return hipGetLastError();
}

// act2 = silu(gate) * up with gu = [gate | up] per row
__global__ void silu_mul_kernel(const float* __restrict__ gu, int d_ffn, float* __restrict__ act2) {
  const int r = blockIdx.y;
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= d_ffn) return;
  const float g = gu[(size_t)r * 2 * d_ffn + j], u = gu[(size_t)r * 2 * d_ffn + d_ffn + j];
  act2[(size_t)r * d_ffn + j] = (g / (1.0f + expf(-g))) * u;
}

hipError_t launch_silu_mul(const float* gu, int m, int d_ffn, float* act2, hipStream_t st) {
  dim3 grid((d_ffn + 255) / 256, m);
  silu_mul_kernel<<<grid, 256, 0, st>>>(gu, d_ffn, act2);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// In-place KV truncation: the rows of the rejected drafts are cleared in every layer, so nothing
// of a rejected suffix survives in the cache (rollback to the last accepted token, Appendix B).
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ void kv_trim_kernel(KvView kv, int first_pos, int k, const int32_t* __restrict__ result) {
  const int a = result[0];
  const int j = blockIdx.x;  // draft row index 1..k -> position first_pos + j
  const int layer = blockIdx.y;
  if (j + 1 <= a) return;    // draft j+1 accepted
  const int pos = first_pos + j + 1;
  T* p = (T*)kv.pool;
  const int kvd = kv.n_kv_heads * kv.head_dim;
  for (int i = threadIdx.x; i < kvd; i += blockDim.x) {
    const int kvh = i / kv.head_dim, e = i % kv.head_dim;
    p[k_index(kv, layer, pos, kvh, e)] = (T)0;
    p[v_index(kv, layer, pos, kvh, e)] = (T)0;
  }
}

hipError_t launch_kv_trim(int dtype, const KvView& kv, int n_layers, int first_pos, int k, const int32_t* result,
                          hipStream_t st) {
  if (k <= 0) return hipSuccess;
  dim3 grid(k, n_layers);
  if (dtype == PIPESD_F32)
    kv_trim_kernel<float><<<grid, 256, 0, st>>>(kv, first_pos, k, result);
  else
    kv_trim_kernel<uint16_t><<<grid, 256, 0, st>>>(kv, first_pos, k, result);
  return hipGetLastError();
}

// grid (draft rows of the longest client, layers, clients)
template <typename T>
__global__ void kv_trim_batch_kernel(KvView kv, TrimBatch b, const int32_t* __restrict__ result) {
  const TrimClient c = b.c[blockIdx.z];
  const int a = result[2 * c.slot];
  const int j = blockIdx.x;
  const int layer = blockIdx.y;
  if (j >= c.k || j + 1 <= a) return;
  kv.table += c.table_off;
  const int pos = c.first_pos + j + 1;
  T* p = (T*)kv.pool;
  const int kvd = kv.n_kv_heads * kv.head_dim;
  for (int i = threadIdx.x; i < kvd; i += blockDim.x) {
    const int kvh = i / kv.head_dim, e = i % kv.head_dim;
    p[k_index(kv, layer, pos, kvh, e)] = (T)0;
    p[v_index(kv, layer, pos, kvh, e)] = (T)0;
  }
}

hipError_t launch_kv_trim_batch(int dtype, const KvView& kv, int n_layers, const TrimBatch& b, const int32_t* result,
                                hipStream_t st) {
  if (b.n < 1 || b.n > kMaxPassClients) return hipErrorInvalidValue;
  int max_k = 0;
  for (int i = 0; i < b.n; ++i) max_k = b.c[i].k > max_k ? b.c[i].k : max_k;
  if (max_k <= 0) return hipSuccess;
  dim3 grid(max_k, n_layers, b.n);
  if (dtype == PIPESD_F32)
    kv_trim_batch_kernel<float><<<grid, 256, 0, st>>>(kv, b, result);
  else
    kv_trim_batch_kernel<uint16_t><<<grid, 256, 0, st>>>(kv, b, result);
  return hipGetLastError();
}

struct TableEntries {
  int32_t v[16];
};
__global__ void set_table_kernel(int32_t* table, int first, TableEntries e, int n) {
  if ((int)threadIdx.x < n) table[first + threadIdx.x] = e.v[threadIdx.x];
}

hipError_t launch_set_table(int32_t* table, int first, const int32_t* entries, int n, hipStream_t st) {
  for (int i = 0; i < n; i += 16) {
    TableEntries e;
    const int c = (n - i < 16) ? (n - i) : 16;
    for (int j = 0; j < 16; ++j) e.v[j] = j < c ? entries[i + j] : 0;
    set_table_kernel<<<1, 64, 0, st>>>(table, first + i, e, c);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
  }
  return hipSuccess;
}

__global__ void chain_step_kernel(int32_t* result, int32_t* result_copy, int k, int guess, const int32_t* alive_in,
                                  int32_t* alive_out) {
  if (threadIdx.x != 0) return;
  const bool alive = alive_in == nullptr || *alive_in != 0;
  if (!alive) {
    result[0] = result[1] = -1;
    if (result_copy != nullptr) result_copy[0] = result_copy[1] = -1;
  }
  if (alive_out != nullptr) *alive_out = (alive && result[0] == k && result[1] == guess) ? 1 : 0;
}

hipError_t launch_chain_step(int32_t* result, int32_t* result_copy, int k, int guess, const int32_t* alive_in,
                             int32_t* alive_out, hipStream_t st) {
  chain_step_kernel<<<1, 64, 0, st>>>(result, result_copy, k, guess, alive_in, alive_out);
  return hipGetLastError();
}

__global__ void clear_words_kernel(unsigned* words, int n) {
  for (int i = threadIdx.x; i < n; i += blockDim.x) words[i] = 0u;
}

hipError_t launch_clear_words(unsigned* words, int n, hipStream_t st) {
  if (n < 1) return hipSuccess;
  clear_words_kernel<<<1, 64, 0, st>>>(words, n);
  return hipGetLastError();
}

}  // namespace pipesd
