// Vocabulary-wide decision of a NAV pass: softmax of the k + 1 logit rows, the accept tests
// u_i < min(1, p_i(d_i)/q_i(d_i)), and the corrected / extra token drawn from max(0, p - q) or
// p_{k+1} (Sec. 2.2: accept what matches, correct the first mismatch; Appendix B: the extra token
// after full acceptance; Sec. 1: the target's output distribution is preserved).
//
// The draw is an integer inverse CDF: weights floor(w * 2^40) are summed as 64-bit integers, which
// is associative, so the parallel scan returns the same index as a sequential one.
#include "common.h"

namespace pipesd {

constexpr int kVThreads = 256;
constexpr int kStatChunks = 64;   // softmax partials per row
constexpr int kScanBlocks = 64;   // workgroups of the CDF scan

struct Uniforms {
  float u[kMaxRows];
};

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float wave_sumf(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ unsigned long long shfl_u64(unsigned long long v, int src) {
  unsigned lo = (unsigned)v, hi = (unsigned)(v >> 32);
  lo = __shfl(lo, src, 64);
  hi = __shfl(hi, src, 64);
  return ((unsigned long long)hi << 32) | lo;
}
__device__ __forceinline__ unsigned long long shfl_up_u64(unsigned long long v, int d) {
  unsigned lo = (unsigned)v, hi = (unsigned)(v >> 32);
  lo = __shfl_up(lo, d, 64);
  hi = __shfl_up(hi, d, 64);
  return ((unsigned long long)hi << 32) | lo;
}

// ------------------------------------------------------------------------------------------
// softmax: per (row, chunk) max and sum of exp; p = exp(z - M) / S with M, S merged from the chunk
// partials in index order is formed where it is used (spec_accept_kernel), never written out
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kVThreads) void softmax_stats_kernel(const float* __restrict__ z, int V,
                                                                  float* __restrict__ stats) {
  __shared__ float red[kVThreads / 64];
  const int row = blockIdx.y, c = blockIdx.x;
  const int per = (V + kStatChunks - 1) / kStatChunks;
  const int lo = c * per, hi = min(V, lo + per);
  const float* zr = z + (size_t)row * V;
  float mx = -INFINITY;
  for (int i = lo + threadIdx.x; i < hi; i += kVThreads) mx = fmaxf(mx, zr[i]);
  mx = wave_max(mx);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  __syncthreads();
  float s = 0.f;
  for (int i = lo + threadIdx.x; i < hi; i += kVThreads) s += expf(zr[i] - mx);
  s = wave_sumf(s);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    stats[((size_t)row * kStatChunks + c) * 2 + 0] = mx;
    stats[((size_t)row * kStatChunks + c) * 2 + 1] = (red[0] + red[1]) + (red[2] + red[3]);
  }
}

hipError_t launch_softmax_stats(const VerifyCall& c, hipStream_t st) {
  dim3 grid(kStatChunks, c.k + 1);
  softmax_stats_kernel<<<grid, kVThreads, 0, st>>>(c.logits_or_p, c.V, c.row_stats);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// decision on probabilities
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ bool accept_test(float p, float q, float u) {
  if (p == 0.f && q == 0.f) return false;  // 0/0 rejects
  const float ratio = p / q;               // correctly rounded fp32 division
  return u < fminf(1.0f, ratio);
}

__device__ __forceinline__ unsigned long long fixed_weight(float p, float q, bool residual) {
  const float w = residual ? fmaxf(0.0f, p - q) : p;
  return (unsigned long long)((double)w * 1099511627776.0);  // floor(w * 2^40), exact
}

__device__ __forceinline__ unsigned long long block_sum_u64(unsigned long long v, unsigned long long* red) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += shfl_u64(v, (threadIdx.x & 63) ^ o);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return red[0] + red[1] + red[2] + red[3];
}

// `stats` == nullptr: `p` holds probabilities.  Otherwise `p` holds logits and `stats` the (max,
// sum of exp) chunk partials of softmax_stats_kernel: the probabilities are formed on the fly by the
// very expressions softmax_write_kernel uses, so the decision is the one the two-step path takes.
// (drafts[0..k-1] and un[0..k] may point into kernel arguments)
__device__ __forceinline__ void spec_accept_body(const float* __restrict__ p, const float* __restrict__ q,
                                                 const float* __restrict__ stats, int k, int V, const int32_t* drafts,
                                                 const float* un, unsigned long long* partial, unsigned* counter,
                                                 int32_t* __restrict__ result, int32_t* __restrict__ result_copy) {
  __shared__ unsigned long long red[kVThreads / 64];
  __shared__ int s_a, s_last;
  __shared__ float s_M[kMaxRows], s_S[kMaxRows];
  const int tid = threadIdx.x;
  const bool from_logits = stats != nullptr;
  __shared__ int s_ok[kMaxRows];
  // Row statistics: one wave per row, lane j holding chunk j's (max, sum of exp); the row's max and
  // the rescaled sum are folded across the wave in a fixed butterfly order.  Every workgroup does
  // this for all k + 1 rows itself (one 512-byte load per row).
  static_assert(kStatChunks == 64, "one chunk partial per lane");
  if (from_logits) {
    const int sper = (V + kStatChunks - 1) / kStatChunks;
    const int lane = tid & 63;
    for (int row = tid >> 6; row <= k; row += kVThreads / 64) {
      const bool have = lane * sper < V;
      const float2 ms = have ? *(const float2*)(stats + ((size_t)row * kStatChunks + lane) * 2) : make_float2(-INFINITY, 0.f);
      float M = ms.x;
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) M = fmaxf(M, __shfl_xor(M, o, 64));
      float S = have ? ms.y * expf(ms.x - M) : 0.f;
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) S += __shfl_xor(S, o, 64);
      if (lane == 0) {
        s_M[row] = M;
        s_S[row] = S;
      }
    }
  }
  __syncthreads();
  if (tid < k) {  // the k tests side by side
    const int d = drafts[tid];
    const float v = p[(size_t)tid * V + d];
    s_ok[tid] = accept_test(from_logits ? expf(v - s_M[tid]) / s_S[tid] : v, q[(size_t)tid * V + d], un[tid]) ? 1 : 0;
  }
  __syncthreads();
  auto prob = [&](int row, int i) -> float {
    const float v = p[(size_t)row * V + i];
    return from_logits ? expf(v - s_M[row]) / s_S[row] : v;
  };
  if (tid == 0) {  // the tests count in order, up to the first failure
    int a = 0;
    while (a < k && s_ok[a]) ++a;
    s_a = a;
  }
  __syncthreads();
  const int a = s_a;
  const bool residual = a < k;
  const float* qr = q + (size_t)(residual ? a : 0) * V;

  const int per = (V + kScanBlocks - 1) / kScanBlocks;
  const int lo = blockIdx.x * per, hi = min(V, lo + per);
  unsigned long long s = 0;
  for (int i = lo + tid; i < hi; i += kVThreads) s += fixed_weight(prob(a, i), residual ? qr[i] : 0.f, residual);
  s = block_sum_u64(s, red);
  if (tid == 0) {
    partial[blockIdx.x] = s;
    __threadfence();
    const unsigned prev = atomicAdd(counter, 1u);
    s_last = (prev == (unsigned)gridDim.x - 1);
  }
  __syncthreads();
  if (!s_last) return;
  __threadfence();
  if (tid >= 64) return;  // the last workgroup's first wave finishes the draw

  unsigned long long W = 0;
  for (int b = 0; b < kScanBlocks; ++b) W += partial[b];
  int next;
  if (W == 0) {
    // every weight truncated to zero: lowest-index maximum of the target row
    float best = -INFINITY;
    int bi = 0x7fffffff;
    for (int i = tid; i < V; i += 64) {
      const float v = prob(a, i);
      if (v > best) { best = v; bi = i; }
    }
    for (int o = 32; o > 0; o >>= 1) {
      const float ob = __shfl_xor(best, o, 64);
      const int oi = __shfl_xor(bi, o, 64);
      if (ob > best || (ob == best && oi < bi)) { best = ob; bi = oi; }
    }
    next = bi;
  } else {
    const unsigned long long ui = (unsigned long long)(un[k] * 16777216.0f);  // floor(u * 2^24)
    const unsigned long long T = (__umul64hi(W, ui) << 40) | ((W * ui) >> 24);
    // chunk whose running total first exceeds T
    unsigned long long run = 0;
    int b = 0;
    for (; b < kScanBlocks - 1; ++b) {
      const unsigned long long nb = run + partial[b];
      if (nb > T) break;
      run = nb;
    }
    const int clo = b * per, chi = min(V, clo + per);
    next = chi - 1;
    bool found = false;
    for (int base = clo; base < chi && !found; base += 64) {
      const int i = base + tid;
      unsigned long long w = (i < chi) ? fixed_weight(prob(a, i), residual ? qr[i] : 0.f, residual) : 0ull;
      unsigned long long inc = w;  // inclusive scan across the wave
#pragma unroll
      for (int d = 1; d < 64; d <<= 1) {
        const unsigned long long o = shfl_up_u64(inc, d);
        if (tid >= d) inc += o;
      }
      const bool hit = (run + inc) > T;
      const unsigned long long m = __ballot(hit);
      if (m != 0ull) {
        next = base + __ffsll((long long)m) - 1;
        found = true;
      } else {
        run += shfl_u64(inc, 63);
      }
    }
  }
  if (tid == 0) {
    result[0] = a;
    result[1] = next;
    if (result_copy != nullptr) {
      result_copy[0] = a;
      result_copy[1] = next;
    }
    *counter = 0u;
  }
}

__global__ __launch_bounds__(kVThreads) void spec_accept_kernel(const float* __restrict__ p, const float* __restrict__ q,
                                                                const float* __restrict__ stats, int k, int V,
                                                                RowTokens drafts, Uniforms un, unsigned long long* partial,
                                                                unsigned* counter, int32_t* __restrict__ result,
                                                                int32_t* __restrict__ result_copy) {
  spec_accept_body(p, q, stats, k, V, drafts.tok, un.u, partial, counter, result, result_copy);
}

hipError_t launch_spec_accept(const VerifyCall& c, hipStream_t st) {
  Uniforms un;
  for (int i = 0; i < kMaxRows; ++i) un.u[i] = c.u[i];
  spec_accept_kernel<<<kScanBlocks, kVThreads, 0, st>>>(c.logits_or_p, c.q, c.from_logits ? c.row_stats : nullptr, c.k,
                                                        c.V, c.drafts, un, c.scan_partial,
                                                        c.counter, c.result, c.result_copy);
  return hipGetLastError();
}

// The decisions of all clients of a pass in one launch: workgroups (scan block, client).  Client ci
// owns logits rows row_off .. row_off + k of the pass, partial sums [ci][kScanBlocks], counter ci and
// result slots 2 slot, 2 slot + 1; its drafts and uniforms sit at the indices of its rows.  Each client
// is decided by the very code of the single-client kernel.
__global__ __launch_bounds__(kVThreads) void spec_accept_batch_kernel(const float* __restrict__ logits,
                                                                      const float* __restrict__ stats, int V,
                                                                      DecisionBatch b, unsigned long long* partial,
                                                                      unsigned* counter, int32_t* __restrict__ result,
                                                                      int32_t* __restrict__ result_copy) {
  const int ci = blockIdx.y;
  const DecisionClient c = b.c[ci];
  spec_accept_body(logits + (size_t)c.row_off * V, c.q, stats + (size_t)c.row_off * kStatChunks * 2, c.k, V,
                   b.drafts.tok + c.row_off, b.u + c.row_off, partial + (size_t)ci * kScanBlocks, counter + ci,
                   result + 2 * c.slot, result_copy ? result_copy + 2 * c.slot : nullptr);
}

hipError_t launch_spec_accept_batch(const DecisionCall& c, hipStream_t st) {
  if (c.batch.n < 1 || c.batch.n > kMaxPassClients || c.rows < 1 || c.rows > kMaxPassRows) return hipErrorInvalidValue;
  for (int i = 0; i < c.batch.n; ++i) {
    const DecisionClient& d = c.batch.c[i];
    if (d.q == nullptr || d.k < 1 || d.k > kMaxRows - 1 || d.row_off < 0 || d.row_off + d.k + 1 > c.rows || d.slot < 0)
      return hipErrorInvalidValue;
  }
  softmax_stats_kernel<<<dim3(kStatChunks, c.rows), kVThreads, 0, st>>>(c.logits, c.V, c.row_stats);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  spec_accept_batch_kernel<<<dim3(kScanBlocks, c.batch.n), kVThreads, 0, st>>>(
      c.logits, c.row_stats, c.V, c.batch, c.scan_partial, c.counter, c.result, c.result_copy);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// token matching on logits: per (row, chunk) argmax, then one workgroup decides
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kVThreads) void argmax_partial_kernel(const float* __restrict__ z, int V,
                                                                   float* __restrict__ stats) {
  __shared__ float rb[kVThreads / 64];
  __shared__ int ri[kVThreads / 64];
  const int row = blockIdx.y, c = blockIdx.x;
  const int per = (V + kStatChunks - 1) / kStatChunks;
  const int lo = c * per, hi = min(V, lo + per);
  const float* zr = z + (size_t)row * V;
  float best = -INFINITY;
  int bi = 0x7fffffff;
  for (int i = lo + threadIdx.x; i < hi; i += kVThreads) {
    const float v = zr[i];
    if (v > best) { best = v; bi = i; }
  }
  for (int o = 32; o > 0; o >>= 1) {
    const float ob = __shfl_xor(best, o, 64);
    const int oi = __shfl_xor(bi, o, 64);
    if (ob > best || (ob == best && oi < bi)) { best = ob; bi = oi; }
  }
  if ((threadIdx.x & 63) == 0) { rb[threadIdx.x >> 6] = best; ri[threadIdx.x >> 6] = bi; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < kVThreads / 64; ++w)
      if (rb[w] > best || (rb[w] == best && ri[w] < bi)) { best = rb[w]; bi = ri[w]; }
    stats[((size_t)row * kStatChunks + c) * 2 + 0] = best;
    stats[((size_t)row * kStatChunks + c) * 2 + 1] = __int_as_float(bi);
  }
}

__global__ void greedy_decide_kernel(const float* __restrict__ stats, int k, int V, RowTokens drafts,
                                     int32_t* __restrict__ result, int32_t* __restrict__ result_copy) {
  __shared__ int am[kMaxRows];
  const int per = (V + kStatChunks - 1) / kStatChunks;
  if ((int)threadIdx.x <= k) {
    const float* st = stats + (size_t)threadIdx.x * kStatChunks * 2;
    float best = -INFINITY;
    int bi = 0x7fffffff;
    for (int j = 0; j < kStatChunks; ++j) {
      if (j * per >= V) break;
      const float v = st[j * 2];
      const int idx = __float_as_int(st[j * 2 + 1]);
      if (v > best || (v == best && idx < bi)) { best = v; bi = idx; }
    }
    am[threadIdx.x] = bi;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int a = 0;
    while (a < k && am[a] == drafts.tok[a]) ++a;
    result[0] = a;
    result[1] = am[a];
    if (result_copy != nullptr) {
      result_copy[0] = a;
      result_copy[1] = am[a];
    }
  }
}

hipError_t launch_greedy_accept(const VerifyCall& c, hipStream_t st) {
  dim3 grid(kStatChunks, c.k + 1);
  argmax_partial_kernel<<<grid, kVThreads, 0, st>>>(c.logits_or_p, c.V, c.row_stats);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  greedy_decide_kernel<<<1, 64, 0, st>>>(c.row_stats, c.k, c.V, c.drafts, c.result, c.result_copy);
  return hipGetLastError();
}

}  // namespace pipesd
