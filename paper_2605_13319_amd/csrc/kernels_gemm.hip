// Per-GEMM kernel of the NAV pass: one launch per projection (used for the LM head, for passes with
// more than 16 rows, and for shapes the fused layer kernel does not take).  The device code lives in
// device_gemm.h.
#include <hip/hip_ext.h>

#include "device_gemm.h"

namespace pipesd {

template <int MT, int KSTEPS>
__global__ __launch_bounds__(512) void gemm_bf16_kernel(GemmArgs a) {
  extern __shared__ float lds[];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  // one team per workgroup: all W waves of the workgroup
  const TeamPos tp{(int)blockIdx.x, (int)gridDim.x, w, 0, true};
  u32x4 af[KSTEPS];
  gemm_prefetch<KSTEPS>(a, tp, lane, af);
  gemm_body<MT, KSTEPS, false>(a, tp, 1, a.W, lds, af);
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
  a.res_in = c.res_in;
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
  const size_t lds = gemm_lds_floats(p.tg, p.W, mt, 1) * sizeof(float);
  if (c.ev_start != nullptr && c.ev_stop != nullptr) {
    if (mt == 1)
      hipExtLaunchKernelGGL((gemm_bf16_kernel<1, 16>), dim3(p.grid), dim3(p.W * 64), (uint32_t)lds, st, c.ev_start,
                            c.ev_stop, 0, a);
    else
      hipExtLaunchKernelGGL((gemm_bf16_kernel<2, 8>), dim3(p.grid), dim3(p.W * 64), (uint32_t)lds, st, c.ev_start,
                            c.ev_stop, 0, a);
  } else if (mt == 1) {
    gemm_bf16_kernel<1, 16><<<p.grid, p.W * 64, lds, st>>>(a);
  } else {
    gemm_bf16_kernel<2, 8><<<p.grid, p.W * 64, lds, st>>>(a);
  }
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
