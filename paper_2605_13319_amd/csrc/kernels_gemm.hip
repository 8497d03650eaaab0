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
//  * A workgroup's W waves cover W K slices of the same n-tiles at a time (and, for long K, P
//    such phases one after the other, accumulators kept in registers) and add their 16x16 partial
//    tiles through LDS in a fixed order.  Nothing crosses workgroups: no global partials, no
//    device-scope fences, no floating-point atomics; results are bit-reproducible.
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
  const float* rope_cs;
  KvView kv;
  int lda, m, K, N, ntiles, kst, W, P, tg, ldo, epi, layer, start_pos, n_q_heads;
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

// Loads this wave's activation fragments for K slice `slice` (KSTEPS k-steps of 32 columns): lane
// (c = row, g = k-group) takes 8 consecutive fp32 values per k-step, multiplies by the norm gain if
// one is fused, adds the raw squares to ssq, and splits into bf16 hi + lo.
template <int MT, int KSTEPS>
__device__ __forceinline__ void load_act_frags(const GemmArgs& a, int slice, int c, int g, bf16x8 (&bhi)[MT][KSTEPS],
                                               bf16x8 (&blo)[MT][KSTEPS], float (&ssq)[MT]) {
  const int k0 = slice * KSTEPS * 32;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int row = mt * 16 + c;
    float part = 0.f;
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
          part = fmaf(v[i], v[i], part);
          v[i] *= gv[i];
        }
      }
      split_hi_lo(v, bhi[mt][ks], blo[mt][ks]);
    }
    part += __shfl_xor(part, 16, 64);
    part += __shfl_xor(part, 32, 64);
    ssq[mt] += part;
  }
}

// Work decomposition: K is cut into W * P slices of KSTEPS*32 columns; wave w of a workgroup takes
// slices p*W + w, p = 0..P-1, one phase after the other, for a group of tg n-tiles, keeping its
// running 16x16 sums in its own LDS slots.  After the last phase the W waves' sums are added.  Groups are dealt to workgroups round-robin.  The weight stream of a wave is a
// fixed sequence of 1 KB-per-instruction chunks and the next chunk is always requested while the
// current one is multiplied, also across phase and group boundaries.
template <int MT, int KSTEPS>
__global__ __launch_bounds__(512) void gemm_bf16_kernel(GemmArgs a) {
  extern __shared__ float lds[];
  f32x4* red = (f32x4*)lds;                                     // [tg][W][MT][64]
  float* ssq_lds = lds + (size_t)a.tg * a.W * MT * 64 * 4;      // [W][MT*16]

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int c = lane & 15, g = lane >> 4;
  const int nthreads = a.W * 64;
  const int ngroups = (a.ntiles + a.tg - 1) / a.tg;
  int grp = blockIdx.x;
  if (grp >= ngroups) return;

  const u32x4* wlane = a.wp + lane;
  auto chunk = [&](int tile, int p) { return wlane + ((size_t)tile * a.kst + (size_t)(p * a.W + w) * KSTEPS) * 64; };

  // the weight stream starts first: it does not depend on the activations
  u32x4 af[KSTEPS];
  {
    const u32x4* first = chunk(grp * a.tg, 0);
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) af[ks] = __builtin_nontemporal_load(first + ks * 64);
  }

  bf16x8 bhi[MT][KSTEPS], blo[MT][KSTEPS];
  float ssq[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) ssq[mt] = 0.f;
  if (a.P == 1) load_act_frags<MT, KSTEPS>(a, w, c, g, bhi, blo, ssq);

  for (; grp < ngroups; grp += gridDim.x) {
    const int t0 = grp * a.tg;
    const int nt_g = min(a.tg, a.ntiles - t0);
    if (a.P > 1) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) ssq[mt] = 0.f;
    }
    for (int p = 0; p < a.P; ++p) {
      if (a.P > 1) load_act_frags<MT, KSTEPS>(a, p * a.W + w, c, g, bhi, blo, ssq);
      for (int t = 0; t < nt_g; ++t) {
        const u32x4* nxt = nullptr;
        if (t + 1 < nt_g) nxt = chunk(t0 + t + 1, p);
        else if (p + 1 < a.P) nxt = chunk(t0, p + 1);
        else if (grp + (int)gridDim.x < ngroups) nxt = chunk((grp + (int)gridDim.x) * a.tg, 0);
        f32x4 acc[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
          const bf16x8 av = as_bf16x8(af[ks]);
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) {
            acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, bhi[mt][ks], acc[mt], 0, 0, 0);
            acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, blo[mt][ks], acc[mt], 0, 0, 0);
          }
          if (nxt != nullptr) af[ks] = __builtin_nontemporal_load(nxt + ks * 64);
        }
        // this wave's running sum over its phases lives in its own LDS slot
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          f32x4* slot = red + ((size_t)(t * a.W + w) * MT + mt) * 64 + lane;
          *slot = (p == 0) ? acc[mt] : (*slot + acc[mt]);
        }
      }
    }
    if (a.gain != nullptr && g == 0) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) ssq_lds[w * MT * 16 + mt * 16 + c] = ssq[mt];
    }
    __syncthreads();
    // add the W partial tiles and finish each (row pair, activation row)
    const int npairs = nt_g * MT * 128;
    const float inv_k = 1.0f / (float)a.K;
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
      epilogue_pair(a, t0 + tt, wr, mt * 16 + cc, v0, v1, rstd);
    }
    __syncthreads();  // red is free again
  }
}

// ------------------------------------------------------------------------------------------------
// launch shape
// ------------------------------------------------------------------------------------------------
constexpr int kTmax16 = 7, kTmax32 = 3;  // n-tiles per group at W = 8 (the LDS reduce area stays under 64 KB)

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

GemmPlan plan_gemm(int N, int K, int n_cu) {
  GemmPlan p{};
  p.K = K;
  p.N = N;
  p.ntiles = (N + 15) / 16;
  (void)n_cu;
  return p;
}

static void shape_for(const GemmPlan& base, int m, int n_cu, GemmPlan& p) {
  p = base;
  const int slices = base.K / (m <= 16 ? 512 : 256);
  int W = 1;
  for (int cand = 8; cand >= 1; --cand)
    if (slices % cand == 0) { W = cand; break; }
  p.W = W;
  p.P = slices / W;
  const int slots = n_cu * (8 / W > 0 ? 8 / W : 1);
  const int tmax = (m <= 16 ? kTmax16 : kTmax32) * 8 / W;
  int best_tg = 1;
  long best_cost = -1;
  for (int tg = 1; tg <= tmax; ++tg) {
    const int groups = (p.ntiles + tg - 1) / tg;
    const long rounds = (groups + slots - 1) / slots;
    const long cost = rounds * tg;
    if (best_cost < 0 || cost <= best_cost) { best_cost = cost; best_tg = tg; }
  }
  p.tg = best_tg;
  const int groups = (p.ntiles + p.tg - 1) / p.tg;
  p.grid = groups < slots ? groups : slots;
}

hipError_t launch_gemm_bf16(const GemmCall& c, hipStream_t st) {
  const int n_cu = device_cu_count();
  if (n_cu <= 0) return hipErrorUnknown;
  const int slice = c.m <= 16 ? 512 : 256;
  if (c.m < 1 || c.m > kMaxRows || c.plan.K % slice != 0 || (c.lda & 3) != 0) return hipErrorInvalidValue;
  GemmPlan p;
  shape_for(c.plan, c.m, n_cu, p);
  GemmArgs a{};
  a.wp = (const u32x4*)c.wp;
  a.act = c.act;
  a.gain = c.gain;
  a.out = c.out;
  a.rope_cs = c.rope_cs;
  a.kv = c.kv;
  a.lda = c.lda;
  a.m = c.m;
  a.K = p.K;
  a.N = p.N;
  a.ntiles = p.ntiles;
  a.kst = p.K / 32;
  a.W = p.W;
  a.P = p.P;
  a.tg = p.tg;
  a.ldo = c.ldo;
  a.epi = c.epi;
  a.layer = c.layer;
  a.start_pos = c.start_pos;
  a.n_q_heads = c.n_q_heads;
  a.eps = c.eps;
  const int mt = c.m <= 16 ? 1 : 2;
  const size_t lds = ((size_t)p.tg * p.W * mt * 64 * 4 + (size_t)p.W * mt * 16) * sizeof(float);
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
