// Per-GEMM kernel of the NAV pass: one launch per projection (used for the LM head, for passes with
// more than 16 rows, and for shapes the fused layer kernel does not take).  The device code lives in
// device_gemm.h.
#include <hip/hip_ext.h>

#include <type_traits>

#include "device_gemm.h"

namespace pipesd {

// EPI (the projection's epilogue) is a template parameter: every projection of a layer is a kernel
// of its own name, with only its own epilogue's code and registers.
// and P1 says that every wave has a single K slice (no phases).
template <int KSTEPS, bool NT, int EPI, bool P1>
__global__ __launch_bounds__(512) void gemm_bf16_kernel(GemmArgs a) {
  extern __shared__ float lds[];
  if (a.gate != nullptr && *a.gate == 0) return;  // (uniform: a round of a chain that does not run)
  const int w = threadIdx.x >> 6;
  // One team per workgroup: all W waves of the workgroup.  With rt row tiles the workgroups b,
  // b + 8, .. b + 8 (rt - 1) form a group on the same tiles (16 rows of the pass each): workgroups
  // are dealt to the 8 chiplets round robin, so a group shares an L2 and the weights cross the
  // memory interface once.
  const int b = (int)blockIdx.x, rt = a.row_tiles;
  TeamPos tp{(b / (8 * rt)) * 8 + (b & 7), (int)gridDim.x / rt, w, 0, true};
  tp.row_base = ((b >> 3) % rt) * 16;
  u32x4 af[KSTEPS];
  gemm_body<1, KSTEPS, false, NT, EPI, P1>(a, tp, 1, a.W, lds, af);
}

// ------------------------------------------------------------------------------------------------
// launch shape
// ------------------------------------------------------------------------------------------------
constexpr int kTmax16 = 7;  // n-tiles per group at W = 8 (the LDS reduce area stays under 64 KB)

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

// launch shape for `slots_cu` compute units' worth of teams (a pass of more than 16 rows puts two
// workgroups on every team's tiles, so it plans for half the device)
static void shape_for(int N, int K, int slots_cu, GemmPlan& p) {
  p.K = K;
  p.N = N;
  p.ntiles = (N + 15) / 16;
  const int slices = K / 512;
  int W = 1;
  for (int cand = 8; cand >= 1; --cand)
    if (slices % cand == 0) { W = cand; break; }
  p.W = W;
  p.P = slices / W;
  const int slots = slots_cu * (8 / W > 0 ? 8 / W : 1);
  const int tmax = kTmax16 * 8 / W;
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
  if (c.m < 1 || c.m > kMaxPassRows || c.K % 512 != 0 || c.act_tiles * 16 < c.m) return hipErrorInvalidValue;
  const int row_tiles = (c.m + 15) / 16;
  GemmPlan p;
  shape_for(c.N, c.K, n_cu / row_tiles, p);
  if (row_tiles > 1) p.grid = (p.grid + 7) / 8 * 8 * row_tiles;  // groups are b, b + 8, ..: whole rounds of the 8 chiplets
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
  a.rows = c.rows;
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
  a.row_tiles = row_tiles;
  a.act_tiles = c.act_tiles;
  a.gate = c.gate;
  if (c.gate != nullptr && row_tiles >= kWideMinRowTiles) return hipErrorInvalidValue;  // the wide kernel has no gate
  if (row_tiles >= kWideMinRowTiles && gemm_wide_supported(c.N, c.K, c.act_tiles) &&
      (c.wide_mode == 2 || (c.wide_mode == 0 && gemm_wide_preferred(c.N, c.K, row_tiles))))
    return launch_gemm_wide(c, a, st);
  const size_t lds = gemm_lds_floats(p.tg, p.W, 1, 1) * sizeof(float);
  const bool timed = c.ev_start != nullptr && c.ev_stop != nullptr;
  auto launch = [&](auto kernel) {
    if (timed)
      hipExtLaunchKernelGGL(kernel, dim3(p.grid), dim3(p.W * 64), (uint32_t)lds, st, c.ev_start, c.ev_stop, 0, a);
    else
      kernel<<<p.grid, p.W * 64, lds, st>>>(a);
  };
  auto launch_p = [&](auto nt, auto p1) {
    constexpr bool NT = decltype(nt)::value, P1 = decltype(p1)::value;
    switch (c.epi) {
      case EPI_STORE: launch(gemm_bf16_kernel<16, NT, EPI_STORE, P1>); break;
      case EPI_RESID: launch(gemm_bf16_kernel<16, NT, EPI_RESID, P1>); break;
      case EPI_SWIGLU: launch(gemm_bf16_kernel<16, NT, EPI_SWIGLU, P1>); break;
      default: launch(gemm_bf16_kernel<16, NT, EPI_QKV, P1>); break;
    }
  };
  auto launch_nt = [&](auto nt) {
    if (p.P == 1)
      launch_p(nt, std::true_type{});
    else
      launch_p(nt, std::false_type{});
  };
  if (c.epi < EPI_STORE || c.epi > EPI_QKV) return hipErrorInvalidValue;
  // the residual epilogue is the one without a fused norm in front of it (compile-time knowledge of the kernels)
  if ((c.ssq_in != nullptr) != (c.epi != EPI_RESID)) return hipErrorInvalidValue;
  if (c.ssq_in != nullptr && c.ssq_parts > 64 * kSsqPerLane) return hipErrorInvalidValue;
  if (row_tiles == 1)
    launch_nt(std::true_type{});
  else
    launch_nt(std::false_type{});
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
