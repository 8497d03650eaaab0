// Skinny GEMM of a NAV pass on the gfx950 matrix cores: y[m][N] = act[m][K] * W[N][K]^T with
// m = k + 1 <= 32 rows (the QKV / O / SwiGLU-FFN / LM-head products of the target forward, Sec. 2.2).
//
// The pass is bound by streaming W once from HBM, so everything is arranged around that stream:
//  * W is re-tiled once, at model creation, into the order the matrix cores consume it: tile
//    (n-tile of 16 weight rows, k-step of 32 columns) is 1 KB, lane l holding row l%16, columns
//    8*(l/16)..+7.  A wave's load instruction then reads 1 KB contiguous and the data lands directly
//    in MFMA operand registers: no LDS pass, no barrier in the main loop.
//  * W is the A operand (16 weight rows x 32 k), the activations are the B operand (32 k x 16 rows).
//    Each wave owns one K slice; its activation fragments stay in registers for the whole kernel,
//    as a bf16 hi + lo pair so that no activation precision is lost (two MFMAs per weight fragment;
//    the matrix cores idle otherwise).
//  * A workgroup's W waves cover W consecutive K slices of the same n-tiles and add their 16x16
//    partial tiles through LDS; if the GEMM is further split over S workgroups along K, the
//    partial tiles go through a global scratch and the last workgroup to arrive adds them in a fixed
//    order.  No floating-point atomics: results are bit-reproducible.
//  * RMSNorm is fused: the kernel multiplies the activations by the gain on load, accumulates
//    sum(x^2) of the raw activations on the way, and scales the finished tile by rstd per row.
//  * Epilogues: plain store (logits), residual add, SiLU(gate)*up, or rotary + query buffer / paged
//    KV-cache append.  Rows 8..15 of a weight tile are the partners of rows 0..7 (other half of the
//    head for the rotary pair; the up-projection row for a gate row) so a pair is finished together.
#include "common.h"

namespace pipesd {

typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

struct GemmArgs {
  const u32x4* wp;
  const float* act;
  const float* gain;
  float* out;
  float* partial;
  float* ssq_partial;
  unsigned* counters;
  const float* rope_cs;
  KvView kv;
  int lda, m, K, N, ntiles, kst, W, S, tpr, nt, ldo, epi, layer, start_pos, n_q_heads;
  float eps;
};

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ __forceinline__ void split_hi_lo(const float (&v)[8], bf16x8& hi, bf16x8& lo) {
  uint32_t h[4], l[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint16_t h0 = f32_to_bf16_bits(v[2 * i]), h1 = f32_to_bf16_bits(v[2 * i + 1]);
    const uint16_t l0 = f32_to_bf16_bits(v[2 * i] - bf16_bits_to_f32(h0));
    const uint16_t l1 = f32_to_bf16_bits(v[2 * i + 1] - bf16_bits_to_f32(h1));
    h[i] = (uint32_t)h0 | ((uint32_t)h1 << 16);
    l[i] = (uint32_t)l0 | ((uint32_t)l1 << 16);
  }
  hi = as_bf16x8(u32x4{h[0], h[1], h[2], h[3]});
  lo = as_bf16x8(u32x4{l[0], l[1], l[2], l[3]});
}

__device__ __forceinline__ void epilogue_pair(const GemmArgs& a, int t, int wr, int row, float v0, float v1,
                                              float rstd) {
  if (row >= a.m) return;
  switch (a.epi) {
    case EPI_STORE: {
      const int n0 = t * 16 + wr, n1 = n0 + 8;
      if (n0 < a.N) a.out[(size_t)row * a.ldo + n0] = v0 * rstd;
      if (n1 < a.N) a.out[(size_t)row * a.ldo + n1] = v1 * rstd;
      break;
    }
    case EPI_RESID: {
      const int n0 = t * 16 + wr, n1 = n0 + 8;
      if (n0 < a.N) a.out[(size_t)row * a.ldo + n0] += v0;
      if (n1 < a.N) a.out[(size_t)row * a.ldo + n1] += v1;
      break;
    }
    case EPI_SWIGLU: {
      const int j = t * 8 + wr;
      const float gt = v0 * rstd, up = v1 * rstd;
      a.out[(size_t)row * a.ldo + j] = (gt / (1.0f + expf(-gt))) * up;
      break;
    }
    case EPI_QKV: {
      const int h = a.kv.head_dim, half = h >> 1, hpt = h >> 4;
      const int hd = t / hpt, i = (t % hpt) * 8 + wr;
      const float x0 = v0 * rstd, x1 = v1 * rstd;
      if (hd < a.n_q_heads + a.kv.n_kv_heads) {
        const float c = a.rope_cs[((size_t)row * half + i) * 2], s = a.rope_cs[((size_t)row * half + i) * 2 + 1];
        const float r0 = x0 * c - x1 * s, r1 = x1 * c + x0 * s;
        if (hd < a.n_q_heads) {
          a.out[(size_t)row * a.ldo + hd * h + i] = r0;
          a.out[(size_t)row * a.ldo + hd * h + i + half] = r1;
        } else {
          uint16_t* pool = (uint16_t*)a.kv.pool;
          const int kvh = hd - a.n_q_heads;
          pool[k_index(a.kv, a.layer, a.start_pos + row, kvh, i)] = f32_to_bf16_bits(r0);
          pool[k_index(a.kv, a.layer, a.start_pos + row, kvh, i + half)] = f32_to_bf16_bits(r1);
        }
      } else {
        uint16_t* pool = (uint16_t*)a.kv.pool;
        const int kvh = hd - a.n_q_heads - a.kv.n_kv_heads;
        pool[v_index(a.kv, a.layer, a.start_pos + row, kvh, i)] = f32_to_bf16_bits(x0);
        pool[v_index(a.kv, a.layer, a.start_pos + row, kvh, i + half)] = f32_to_bf16_bits(x1);
      }
      break;
    }
  }
}

template <int MT, int KSTEPS>
__global__ __launch_bounds__(512) void gemm_bf16_kernel(GemmArgs a) {
  extern __shared__ float lds[];
  // red[nt][W][MT][64] float4, then ssq[W][MT*16], then one flag
  f32x4* red = (f32x4*)lds;
  float* ssq_lds = lds + (size_t)a.nt * a.W * MT * 64 * 4;
  int* flag = (int*)(ssq_lds + a.W * MT * 16);

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int c = lane & 15, g = lane >> 4;
  const int s = blockIdx.x % a.S, ri = blockIdx.x / a.S;
  const int k0 = (s * a.W + w) * KSTEPS * 32;
  const int t_begin = ri * a.tpr, t_end = min(a.ntiles, t_begin + a.tpr);
  const int nthreads = a.W * 64;

  // the weight stream starts first: it does not depend on the activations
  const u32x4* wlane = a.wp + (size_t)(k0 / 32) * 64 + lane;
  u32x4 af[KSTEPS];
  if (t_begin < t_end) {
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks)
      af[ks] = __builtin_nontemporal_load(wlane + ((size_t)t_begin * a.kst + ks) * 64);
  }

  // activation fragments of this wave's K slice, kept for the whole kernel
  bf16x8 bhi[MT][KSTEPS], blo[MT][KSTEPS];
  float ssq[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    ssq[mt] = 0.f;
    const int row = mt * 16 + c;
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) {
      const int kk = k0 + ks * 32 + g * 8;
      float v[8];
      if (row < a.m) {
        const float4 x0 = *(const float4*)(a.act + (size_t)row * a.lda + kk);
        const float4 x1 = *(const float4*)(a.act + (size_t)row * a.lda + kk + 4);
        v[0] = x0.x; v[1] = x0.y; v[2] = x0.z; v[3] = x0.w;
        v[4] = x1.x; v[5] = x1.y; v[6] = x1.z; v[7] = x1.w;
      } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = 0.f;
      }
      if (a.gain != nullptr) {
        const float4 g0 = *(const float4*)(a.gain + kk), g1 = *(const float4*)(a.gain + kk + 4);
        const float gv[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          ssq[mt] = fmaf(v[i], v[i], ssq[mt]);
          v[i] *= gv[i];
        }
      }
      split_hi_lo(v, bhi[mt][ks], blo[mt][ks]);
    }
    ssq[mt] += __shfl_xor(ssq[mt], 16, 64);
    ssq[mt] += __shfl_xor(ssq[mt], 32, 64);
    if (g == 0) ssq_lds[w * MT * 16 + mt * 16 + c] = ssq[mt];
  }

  int nb = 0;
  for (int t = t_begin; t < t_end; ++t) {
    f32x4 acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
    const bool more = t + 1 < t_end;
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) {
      const bf16x8 av = as_bf16x8(af[ks]);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, bhi[mt][ks], acc[mt], 0, 0, 0);
        acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, blo[mt][ks], acc[mt], 0, 0, 0);
      }
      if (more) af[ks] = __builtin_nontemporal_load(wlane + ((size_t)(t + 1) * a.kst + ks) * 64);
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) red[((size_t)(nb * a.W + w) * MT + mt) * 64 + lane] = acc[mt];
    ++nb;
    if (nb < a.nt && more) continue;

    // ---- add the W partial tiles of this batch and finish (or hand over to the last arriver) ----
    const int t_first = t - nb + 1;
    const int npairs = nb * MT * 128;
    const float inv_k = 1.0f / (float)a.K;
    __syncthreads();
    if (a.S == 1) {
      for (int e = tid; e < npairs; e += nthreads) {
        const int tt = e / (MT * 128), rem = e % (MT * 128), mt = rem / 128, pr = rem % 128;
        const int wr = pr >> 4, cc = pr & 15;
        const int l0 = (wr >> 2) * 16 + cc, comp = wr & 3;
        float v0 = 0.f, v1 = 0.f;
        for (int ww = 0; ww < a.W; ++ww) {
          const float* rp = (const float*)(red + ((size_t)(tt * a.W + ww) * MT + mt) * 64);
          v0 += rp[l0 * 4 + comp];
          v1 += rp[(l0 + 32) * 4 + comp];
        }
        float rstd = 1.0f;
        if (a.gain != nullptr) {
          float q = 0.f;
          for (int ww = 0; ww < a.W; ++ww) q += ssq_lds[ww * MT * 16 + mt * 16 + cc];
          rstd = 1.0f / sqrtf(q * inv_k + a.eps);
        }
        epilogue_pair(a, t_first + tt, wr, mt * 16 + cc, v0, v1, rstd);
      }
    } else {
      const int bpr = (a.tpr + a.nt - 1) / a.nt;
      const int cidx = ri * bpr + (t_first - t_begin) / a.nt;
      for (int e = tid; e < npairs; e += nthreads) {
        const int tt = e / (MT * 128), rem = e % (MT * 128), mt = rem / 128, pr = rem % 128;
        const int wr = pr >> 4, cc = pr & 15;
        const int l0 = (wr >> 2) * 16 + cc, comp = wr & 3;
        float v0 = 0.f, v1 = 0.f;
        for (int ww = 0; ww < a.W; ++ww) {
          const float* rp = (const float*)(red + ((size_t)(tt * a.W + ww) * MT + mt) * 64);
          v0 += rp[l0 * 4 + comp];
          v1 += rp[(l0 + 32) * 4 + comp];
        }
        float2* dst = (float2*)(a.partial + ((((size_t)s * a.ntiles + t_first + tt) * MT + mt) * 128 + pr) * 2);
        *dst = make_float2(v0, v1);
      }
      if (a.gain != nullptr && tid < MT * 16) {
        float q = 0.f;
        for (int ww = 0; ww < a.W; ++ww) q += ssq_lds[ww * MT * 16 + tid];
        a.ssq_partial[((size_t)cidx * a.S + s) * 32 + tid] = q;
      }
      __threadfence();
      __syncthreads();
      if (tid == 0) {
        const unsigned prev = atomicAdd(a.counters + cidx, 1u);
        *flag = (prev == (unsigned)a.S - 1u) ? 1 : 0;
      }
      __syncthreads();
      if (*flag) {
        __threadfence();
        for (int e = tid; e < npairs; e += nthreads) {
          const int tt = e / (MT * 128), rem = e % (MT * 128), mt = rem / 128, pr = rem % 128;
          const int wr = pr >> 4, cc = pr & 15;
          float v0 = 0.f, v1 = 0.f;
          for (int ss = 0; ss < a.S; ++ss) {
            const float2 pv =
                *(const float2*)(a.partial + ((((size_t)ss * a.ntiles + t_first + tt) * MT + mt) * 128 + pr) * 2);
            v0 += pv.x;
            v1 += pv.y;
          }
          float rstd = 1.0f;
          if (a.gain != nullptr) {
            float q = 0.f;
            for (int ss = 0; ss < a.S; ++ss) q += a.ssq_partial[((size_t)cidx * a.S + ss) * 32 + mt * 16 + cc];
            rstd = 1.0f / sqrtf(q * inv_k + a.eps);
          }
          epilogue_pair(a, t_first + tt, wr, mt * 16 + cc, v0, v1, rstd);
        }
        if (tid == 0) a.counters[cidx] = 0u;
      }
    }
    __syncthreads();  // red is free again
    nb = 0;
  }
}

// ------------------------------------------------------------------------------------------------
// launch shape
// ------------------------------------------------------------------------------------------------
static int slice_cols(int m) { return m <= 16 ? 512 : 256; }

GemmPlan plan_gemm(int N, int K, int n_cu) {
  // planned for the 16-row variant; launch_gemm_bf16 re-derives W and S for the 32-row variant
  GemmPlan p{};
  p.K = K;
  p.N = N;
  p.ntiles = (N + 15) / 16;
  (void)n_cu;
  return p;
}

static void shape_for(const GemmPlan& base, int m, int n_cu, GemmPlan& p) {
  p = base;
  const int nsl = base.K / slice_cols(m);
  int W = 1;
  for (int cand = 8; cand >= 1; --cand)
    if (nsl % cand == 0) { W = cand; break; }
  p.W = W;
  p.S = nsl / W;
  const int wg_per_cu = 8 / W > 0 ? 8 / W : 1;
  int target = n_cu * wg_per_cu;
  int nranges = target / p.S;
  if (nranges < 1) nranges = 1;
  if (nranges > p.ntiles) nranges = p.ntiles;
  p.tpr = (p.ntiles + nranges - 1) / nranges;
  nranges = (p.ntiles + p.tpr - 1) / p.tpr;
  p.grid = nranges * p.S;
  const int nt_max = m <= 16 ? 4 : 2;  // keeps the LDS reduce area under 64 KB
  p.nt = p.tpr < nt_max ? p.tpr : nt_max;
}

// scratch one GEMM shape can need (both row variants): split-K partial tiles, per-batch sum-of-squares
// partials, and arrival counters
void gemm_scratch_need(int N, int K, int n_cu, size_t* partial_floats, size_t* ssq_floats, size_t* counters) {
  *partial_floats = *ssq_floats = *counters = 0;
  for (int m : {16, 32}) {
    GemmPlan base{}, p{};
    base.K = K;
    base.N = N;
    base.ntiles = (N + 15) / 16;
    shape_for(base, m, n_cu, p);
    const int mt = m <= 16 ? 1 : 2;
    const size_t nranges = p.grid / p.S, bpr = (p.tpr + p.nt - 1) / p.nt;
    const size_t pf = p.S > 1 ? (size_t)p.S * p.ntiles * mt * 256 : 0;
    const size_t cn = p.S > 1 ? nranges * bpr : 0;
    if (pf > *partial_floats) *partial_floats = pf;
    if (cn > *counters) *counters = cn;
    if (cn * p.S * 32 > *ssq_floats) *ssq_floats = cn * p.S * 32;
  }
}

int device_cu_count() {
  static int n_cu = 0;
  if (n_cu == 0) {
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return 0;
    n_cu = prop.multiProcessorCount;
  }
  return n_cu;
}

hipError_t launch_gemm_bf16(const GemmCall& c, hipStream_t st) {
  const int n_cu = device_cu_count();
  if (n_cu <= 0) return hipErrorUnknown;
  if (c.m < 1 || c.m > kMaxRows || c.plan.K % slice_cols(c.m) != 0 || (c.lda & 3) != 0) return hipErrorInvalidValue;
  GemmPlan p;
  shape_for(c.plan, c.m, n_cu, p);
  GemmArgs a{};
  a.wp = (const u32x4*)c.wp;
  a.act = c.act;
  a.gain = c.gain;
  a.out = c.out;
  a.partial = c.partial;
  a.ssq_partial = c.ssq_partial;
  a.counters = c.counters;
  a.rope_cs = c.rope_cs;
  a.kv = c.kv;
  a.lda = c.lda;
  a.m = c.m;
  a.K = p.K;
  a.N = p.N;
  a.ntiles = p.ntiles;
  a.kst = p.K / 32;
  a.W = p.W;
  a.S = p.S;
  a.tpr = p.tpr;
  a.nt = p.nt;
  a.ldo = c.ldo;
  a.epi = c.epi;
  a.layer = c.layer;
  a.start_pos = c.start_pos;
  a.n_q_heads = c.n_q_heads;
  a.eps = c.eps;
  const int mt = c.m <= 16 ? 1 : 2;
  const size_t lds = ((size_t)p.nt * p.W * mt * 64 * 4 + (size_t)p.W * mt * 16 + 4) * sizeof(float);
  if (mt == 1)
    gemm_bf16_kernel<1, 16><<<p.grid, p.W * 64, lds, st>>>(a);
  else
    gemm_bf16_kernel<2, 8><<<p.grid, p.W * 64, lds, st>>>(a);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// re-tiling of the caller's row-major weights
// ------------------------------------------------------------------------------------------------
__global__ void pack_bf16_kernel(PackSrc s, int n_src, int K, int mode, int pair_span, uint4* __restrict__ dst,
                                 int ntiles) {
  const int kst = K / 32;
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;  // (tile, kstep, lane)
  const size_t total = (size_t)ntiles * kst * 64;
  if (idx >= total) return;
  const int lane = (int)(idx & 63);
  const int ks = (int)((idx >> 6) % kst);
  const int t = (int)((idx >> 6) / kst);
  const int i = lane & 15, g = lane >> 4;
  long vr;  // row in the stacked sources
  if (mode == PACK_PLAIN) {
    vr = (long)t * 16 + i;
  } else {
    const int tpg = pair_span / 8;  // tiles per group of 2 * pair_span rows
    const long base = (long)(t / tpg) * 2 * pair_span + (long)(t % tpg) * 8;
    vr = i < 8 ? base + i : base + pair_span + (i - 8);
  }
  uint4 v = make_uint4(0, 0, 0, 0);
  for (int j = 0; j < n_src; ++j) {
    if (vr < s.rows[j]) {
      v = *(const uint4*)(s.src[j] + (size_t)vr * K + ks * 32 + g * 8);
      break;
    }
    vr -= s.rows[j];
  }
  dst[idx] = v;
}

hipError_t launch_pack_bf16(const PackSrc& s, int n_src, int K, int mode, int pair_span, void* dst, int ntiles,
                            hipStream_t st) {
  const size_t total = (size_t)ntiles * (K / 32) * 64;
  const unsigned blocks = (unsigned)((total + 255) / 256);
  pack_bf16_kernel<<<blocks, 256, 0, st>>>(s, n_src, K, mode, pair_span, (uint4*)dst, ntiles);
  return hipGetLastError();
}

}  // namespace pipesd
