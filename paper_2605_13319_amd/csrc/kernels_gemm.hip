// Skinny GEMM of a NAV pass on the gfx950 matrix cores: y[m][N] = act[m][K] * W[N][K]^T with
// m = k + 1 <= 32 rows (the QKV / O / SwiGLU-FFN / LM-head products of the target forward, Sec. 2.2).
//
// The pass is bound by streaming W once from HBM, so everything is arranged around that stream:
//  * W is re-tiled once, at model creation, into the order the matrix cores consume it: tile
//    (n-tile of 16 weight rows, k-step of 32 columns) is 1 KB, lane l holding row l%16, columns
//    8*(l/16)..+7.  A wave's load instruction then reads 1 KB contiguous and the data lands directly
//    in MFMA operand registers: no LDS pass, no barrier in the main loop.
//  * W is the A operand (16 weight rows x 32 k), the activations are the B operand (32 k x 16 rows).
//    Activations travel between kernels already in B-operand layout as a bf16 hi + lo pair (see
//    ActPack in common.h): the producing epilogue splits each value once, every consuming wave just
//    loads registers.  Two MFMAs per weight fragment keep 16 significand bits of the activations;
//    the matrix cores idle otherwise.
//  * A workgroup's W waves cover W K slices of the same n-tiles at a time (and, for long K, P
//    such phases one after the other) and add their 16x16 partial tiles through LDS in a fixed
//    order.  Nothing crosses workgroups: no global partials, no device-scope fences, no
//    floating-point atomics; results are bit-reproducible.
//  * RMSNorm is fused: the producer stores x * gain and per-tile sums of x^2; the consumer scales the
//    finished tile by rstd per row.
//  * Epilogues: plain store (logits), residual add (+ packed, gained copy for the next GEMM),
//    SiLU(gate)*up (packed), or rotary + query buffer / paged KV-cache append.  Rows 8..15 of a
//    weight tile are the partners of rows 0..7 (other half of the head for the rotary pair; the
//    up-projection row for a gate row) so a pair is finished by one thread.
#include "common.h"

namespace pipesd {

typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

struct GemmArgs {
  const u32x4* wp;
  const u32x4* actp;      // packed activations (ActPack, K columns)
  const float* ssq_in;    // fused norm: [row][ssq_stride] partial sums of x^2, or nullptr
  int ssq_parts, ssq_stride;
  float* out;             // STORE: logits; RESID: residual stream; QKV: query buffer
  u32x4* outp;            // RESID / SWIGLU: packed output for the next GEMM
  const float* gain_next; // RESID: gain applied to the packed copy
  float* ssq_out;         // RESID: [row][ssq_stride] per-tile sums of x_new^2
  const float* rope_cs;
  KvView kv;
  int m, K, N, ntiles, kst, W, P, tg, ldo, epi, layer, start_pos, n_q_heads;
  float eps;
};

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// The weight stream is issued and awaited by hand: the loads are opaque to the compiler's wait-count
// bookkeeping, and each use is preceded by an explicit s_waitcnt tied to the register it releases.
// Vector memory loads return in order, so "at most N younger loads outstanding" is exact here: the
// compiler would otherwise join the with-next and without-next paths into vmcnt(0) and drain the
// pipeline at every chunk.
__device__ __forceinline__ u32x4 stream_load(const u32x4* p) {
  u32x4 v;
  asm volatile("global_load_dwordx4 %0, %1, off nt" : "=v"(v) : "v"(p));
  return v;
}
__device__ __forceinline__ u32x4 cached_load(const u32x4* p) {
  u32x4 v;
  asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(v) : "v"(p));
  return v;
}
template <int N>
__device__ __forceinline__ void wait_younger(u32x4& v) {
  asm volatile("s_waitcnt vmcnt(%1)" : "+v"(v) : "n"(N));
}

// one chunk = KSTEPS weight fragments of one n-tile against this wave's activation fragments; while
// fragment ks is multiplied, fragment ks of the next chunk is requested into the same registers
template <int MT, int KSTEPS, bool HAS_NEXT, int KS = 0>
__device__ __forceinline__ void chunk_mfma(u32x4 (&af)[KSTEPS], const u32x4 (&bhi)[MT][KSTEPS],
                                           const u32x4 (&blo)[MT][KSTEPS], f32x4 (&acc)[MT], const u32x4* nxt) {
  if constexpr (KS < KSTEPS) {
    wait_younger<HAS_NEXT ? KSTEPS - 1 : KSTEPS - 1 - KS>(af[KS]);
    const bf16x8 av = as_bf16x8(af[KS]);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, as_bf16x8(bhi[mt][KS]), acc[mt], 0, 0, 0);
      acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, as_bf16x8(blo[mt][KS]), acc[mt], 0, 0, 0);
    }
    if constexpr (HAS_NEXT) af[KS] = stream_load(nxt + KS * 64);
    chunk_mfma<MT, KSTEPS, HAS_NEXT, KS + 1>(af, bhi, blo, acc, nxt);
  }
}

__device__ __forceinline__ f32x4 shfl4(f32x4 v, int src) {
  return f32x4{__shfl(v[0], src, 64), __shfl(v[1], src, 64), __shfl(v[2], src, 64), __shfl(v[3], src, 64)};
}

// Finish one n-tile with a whole wave: lane (gg = lane/16, cc = lane%16) holds the dot products of
// activation row `row` with weight rows gg*4 .. gg*4+3 of tile t.  Partner rows (i, i+8) sit 32 lanes
// apart and the two halves of an 8-column group 16 lanes apart, so pairs are joined by shuffles.
// Every lane of the wave must call this (rows beyond the pass only skip the stores).
__device__ __forceinline__ void epilogue_quad(const GemmArgs& a, int t, int row, int lane, f32x4 v, float rstd) {
  const int gg = lane >> 4;
  const bool live = row < a.m;
  switch (a.epi) {
    case EPI_STORE: {
      if (!live) break;
      float* o = a.out + (size_t)row * a.ldo + t * 16 + gg * 4;
      if (t * 16 + 16 <= a.N && (a.ldo & 3) == 0) {
        *(float4*)o = make_float4(v[0] * rstd, v[1] * rstd, v[2] * rstd, v[3] * rstd);
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (t * 16 + gg * 4 + i < a.N) o[i] = v[i] * rstd;
      }
      break;
    }
    case EPI_RESID: {
      float* o = a.out + (size_t)row * a.ldo + t * 16 + gg * 4;
      f32x4 x = f32x4{0.f, 0.f, 0.f, 0.f};
      if (live) {
        const float4 old = *(const float4*)o;
        x = f32x4{old.x + v[0], old.y + v[1], old.z + v[2], old.w + v[3]};
        *(float4*)o = make_float4(x[0], x[1], x[2], x[3]);
      }
      float sq = x[0] * x[0] + x[1] * x[1] + x[2] * x[2] + x[3] * x[3];
      sq += __shfl_xor(sq, 16, 64);
      sq += __shfl_xor(sq, 32, 64);
      const float4 gn = *(const float4*)(a.gain_next + t * 16 + gg * 4);
      const f32x4 y = f32x4{x[0] * gn.x, x[1] * gn.y, x[2] * gn.z, x[3] * gn.w};
      const f32x4 hi4 = shfl4(y, lane + 16);  // columns +4..+7 of the 8-column group
      if (live && (gg & 1) == 0) {
        const float y8[8] = {y[0], y[1], y[2], y[3], hi4[0], hi4[1], hi4[2], hi4[3]};
        store_act8((uint4*)a.outp, row, t * 16 + gg * 4, y8);
        if (gg == 0) a.ssq_out[(size_t)row * a.ssq_stride + t] = sq;
      }
      break;
    }
    case EPI_SWIGLU: {
      const f32x4 up = shfl4(v, lane + 32);
      f32x4 y;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float gt = v[i] * rstd;
        y[i] = (gt / (1.0f + expf(-gt))) * (up[i] * rstd);
      }
      const f32x4 hi4 = shfl4(y, lane + 16);
      if (live && gg == 0) {
        const float y8[8] = {y[0], y[1], y[2], y[3], hi4[0], hi4[1], hi4[2], hi4[3]};
        store_act8((uint4*)a.outp, row, t * 8, y8);
      }
      break;
    }
    case EPI_QKV: {
      const f32x4 x1 = shfl4(v, lane + 32);
      if (!live || gg >= 2) break;
      const int h = a.kv.head_dim, half = h >> 1, hpt = h >> 4;
      const int hd = t / hpt, i0 = (t % hpt) * 8 + gg * 4;
      float r0[4], r1[4];
      if (hd < a.n_q_heads + a.kv.n_kv_heads) {
        const float* cs = a.rope_cs + ((size_t)row * half + i0) * 2;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float p0 = v[i] * rstd, p1 = x1[i] * rstd, c = cs[2 * i], sn = cs[2 * i + 1];
          r0[i] = p0 * c - p1 * sn;
          r1[i] = p1 * c + p0 * sn;
        }
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          r0[i] = v[i] * rstd;
          r1[i] = x1[i] * rstd;
        }
      }
      if (hd < a.n_q_heads) {
        float* o = a.out + (size_t)row * a.ldo + hd * h + i0;
        *(float4*)o = make_float4(r0[0], r0[1], r0[2], r0[3]);
        *(float4*)(o + half) = make_float4(r1[0], r1[1], r1[2], r1[3]);
      } else {
        uint16_t* pool = (uint16_t*)a.kv.pool;
        const int pos = a.start_pos + row;
        if (hd < a.n_q_heads + a.kv.n_kv_heads) {
          const int kvh = hd - a.n_q_heads;
          uint16_t b0[4], b1[4];
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            b0[i] = f32_to_bf16_bits(r0[i]);
            b1[i] = f32_to_bf16_bits(r1[i]);
          }
          *(uint2*)(pool + k_index(a.kv, a.layer, pos, kvh, i0)) = *(const uint2*)b0;
          *(uint2*)(pool + k_index(a.kv, a.layer, pos, kvh, i0 + half)) = *(const uint2*)b1;
        } else {
          const int kvh = hd - a.n_q_heads - a.kv.n_kv_heads;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            pool[v_index(a.kv, a.layer, pos, kvh, i0 + i)] = f32_to_bf16_bits(r0[i]);
            pool[v_index(a.kv, a.layer, pos, kvh, i0 + half + i)] = f32_to_bf16_bits(r1[i]);
          }
        }
      }
      break;
    }
  }
}

// Work decomposition: K is cut into W * P slices of KSTEPS*32 columns; wave w of a workgroup takes
// slices p*W + w, p = 0..P-1, one phase after the other, for a group of tg n-tiles, keeping its
// running 16x16 sums in its own LDS slots.  After the last phase the W waves' sums are added.
// Groups are dealt to workgroups round-robin.  The weight stream of a wave is a fixed sequence of
// 1 KB-per-instruction chunks and the next chunk is always requested while the current one is
// multiplied, also across phase and group boundaries.
template <int MT, int KSTEPS>
__global__ __launch_bounds__(512) void gemm_bf16_kernel(GemmArgs a) {
  extern __shared__ float lds[];
  f32x4* red = (f32x4*)lds;                                     // [tg][W][MT][64]
  float* rstd_lds = lds + (size_t)a.tg * a.W * MT * 64 * 4;     // [MT*16]

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
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
    for (int ks = 0; ks < KSTEPS; ++ks) af[ks] = stream_load(first + ks * 64);
  }

  // activation fragments of the current K slice; loaded by hand too and awaited in full (they and the
  // first weight chunk are all needed before the first MFMA)
  // (lanes whose row is not part of the pass load nothing: their MFMA columns are never stored)
  u32x4 bhi[MT][KSTEPS], blo[MT][KSTEPS];
  const int bc = lane & 15, bg = lane >> 4;
  auto load_act = [&](int slice) {
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        if (mt * 16 + bc < a.m) {
          bhi[mt][ks] = cached_load(a.actp + act_index(slice * KSTEPS + ks, mt, 0, bc, bg));
          blo[mt][ks] = cached_load(a.actp + act_index(slice * KSTEPS + ks, mt, 1, bc, bg));
        }
      }
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        wait_younger<0>(bhi[mt][ks]);
        wait_younger<0>(blo[mt][ks]);
      }
  };
  if (a.P == 1) load_act(w);

  // fused norm: rstd per row from the producer's partial sums of squares, added in index order
  if (a.ssq_in != nullptr) {
    for (int row = w; row < MT * 16; row += a.W) {
      float q = 0.f;
      if (row < a.m)
        for (int j = lane; j < a.ssq_parts; j += 64) q += a.ssq_in[(size_t)row * a.ssq_stride + j];
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) q += __shfl_xor(q, o, 64);
      if (lane == 0) rstd_lds[row] = 1.0f / sqrtf(q / (float)a.K + a.eps);
    }
  }

  for (; grp < ngroups; grp += gridDim.x) {
    const int t0 = grp * a.tg;
    const int nt_g = min(a.tg, a.ntiles - t0);
    for (int p = 0; p < a.P; ++p) {
      if (a.P > 1) load_act(p * a.W + w);
      for (int t = 0; t < nt_g; ++t) {
        const u32x4* nxt = nullptr;
        if (t + 1 < nt_g) nxt = chunk(t0 + t + 1, p);
        else if (p + 1 < a.P) nxt = chunk(t0, p + 1);
        else if (grp + (int)gridDim.x < ngroups) nxt = chunk((grp + (int)gridDim.x) * a.tg, 0);
        f32x4 acc[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (nxt != nullptr)
          chunk_mfma<MT, KSTEPS, true>(af, bhi, blo, acc, nxt);
        else
          chunk_mfma<MT, KSTEPS, false>(af, bhi, blo, acc, nxt);
        // this wave's running sum over its phases lives in its own LDS slot
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          f32x4* slot = red + ((size_t)(t * a.W + w) * MT + mt) * 64 + lane;
          *slot = (p == 0) ? acc[mt] : (*slot + acc[mt]);
        }
      }
    }
    __syncthreads();
    // one lane per 4 tile rows x 1 activation row: add the W partial tiles, then finish with the wave
    const int nquads = nt_g * MT * 64;
    for (int e = tid; e < nquads; e += nthreads) {
      const int tt = e / (MT * 64), rem = e % (MT * 64), mt = rem >> 6, l = rem & 63;
      f32x4 v = f32x4{0.f, 0.f, 0.f, 0.f};
      for (int ww = 0; ww < a.W; ++ww) v += red[((size_t)(tt * a.W + ww) * MT + mt) * 64 + l];
      const int row = mt * 16 + (l & 15);
      const float rstd = (a.ssq_in != nullptr && row < a.m) ? rstd_lds[row] : 1.0f;
      epilogue_quad(a, t0 + tt, row, l, v, rstd);
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

static void shape_for(int N, int K, int m, int n_cu, GemmPlan& p) {
  p.K = K;
  p.N = N;
  p.ntiles = (N + 15) / 16;
  const int slices = K / (m <= 16 ? 512 : 256);
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
  if (c.m < 1 || c.m > kMaxRows || c.K % slice != 0) return hipErrorInvalidValue;
  GemmPlan p;
  shape_for(c.N, c.K, c.m, n_cu, p);
  GemmArgs a{};
  a.wp = (const u32x4*)c.wp;
  a.actp = (const u32x4*)c.actp;
  a.ssq_in = c.ssq_in;
  a.ssq_parts = c.ssq_parts;
  a.ssq_stride = c.ssq_stride;
  a.out = c.out;
  a.outp = (u32x4*)c.outp;
  a.gain_next = c.gain_next;
  a.ssq_out = c.ssq_out;
  a.rope_cs = c.rope_cs;
  a.kv = c.kv;
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
  const size_t lds = ((size_t)p.tg * p.W * mt * 64 * 4 + 32) * sizeof(float);
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
