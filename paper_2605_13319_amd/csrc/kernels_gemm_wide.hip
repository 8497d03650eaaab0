// GEMM for passes of 65..128 rows (batched verification of many clients, prompt ingestion).
//
// At this many rows the activations of a K slice no longer fit a wave's registers, and spreading the
// rows over workgroups that re-read the weights from the L2 (the narrow kernel's way) moves eight
// times the weights through it.  Here a workgroup of four waves multiplies ALL rows of the pass with
// 8 n-tiles of weights: the activations of four k-steps at a time are staged in LDS in the lane
// order the matrix cores consume (double buffered, one barrier per stage; all 8 row tiles of the
// buffers are staged and multiplied, rows past the pass are just never stored), every weight fragment
// comes straight from memory into the A-operand registers of the one pair of waves that needs it,
// and each wave owns a 64-column x 64-row block of the product (4 x 4 accumulator tiles), so every
// LDS read feeds four MFMAs.
//
// Results are bit-identical to the narrow kernel's, row by row: K is cut into the same W * P slices
// of 512 columns, every slice is accumulated from zero in the same k-step order (hi half, then lo
// half of the activations), slices p*W + w are added in the order p = 0..P-1 and the W sums in the
// order w = 0..W-1, starting from zero.  Two ways to get enough workgroups:
//  * WHOLE: a workgroup walks all slices of its columns and finishes them itself (epilogue from the
//    accumulators); chosen when the columns alone fill the device (gate/up, LM head);
//  * split: workgroup (column group, w) walks the P slices of role w only and leaves its running sum
//    in a workspace; a second small kernel adds the W sums in order and runs the epilogue.
#include <hip/hip_ext.h>

#include "device_gemm.h"

namespace pipesd {

constexpr int kWideStage = 4;       // k-steps per LDS stage
constexpr int kWideRowTiles = 8;    // row tiles of the staged activations (= ActPack row tiles of a wide pass)
constexpr int kWideWgTiles = 8;     // n-tiles per workgroup: 2 wave columns x 4
constexpr int kWideAhead = 3;       // blocks of LDS operand reads in flight ahead of the multiplies
constexpr int kWideFrags = kWideStage * kWideRowTiles * 2;  // 1 KB fragments per stage
constexpr size_t kWideLdsBytes = 2 * kWideFrags * 1024 + kWideRowTiles * 16 * sizeof(float);

struct WideArgs {
  f32x4* partials;  // split: [W][ntiles][8][64] running sums of role w
  int ncg;          // column groups of kWideWgTiles n-tiles
  int row_tiles;    // live row tiles of the pass
};

// rstd of the rows row0 + i*row_step, i < NR (one wave; all partial sums are requested before any is
// added), in the narrow kernel's order: lane sums of the partial sums j = lane, lane + 64, .., then
// the xor butterfly 32, 16, .., 1
template <int NR>
__device__ __forceinline__ void wide_rstd_rows(const GemmArgs& a, int row0, int row_step, int lane, float* rstd_lds,
                                               int lds_row0) {
  float v[kSsqPerLane][NR];
#pragma unroll
  for (int j4 = 0; j4 < kSsqPerLane; ++j4)
#pragma unroll
    for (int i = 0; i < NR; ++i) {
      const int row = row0 + i * row_step, j = lane + 64 * j4;
      v[j4][i] = (row < a.m && j < a.ssq_parts) ? a.ssq_in[(size_t)row * a.ssq_stride + j] : 0.f;
    }
#pragma unroll
  for (int i = 0; i < NR; ++i) {
    float t = v[0][i];
#pragma unroll
    for (int j4 = 1; j4 < kSsqPerLane; ++j4) t += v[j4][i];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) t += __shfl_xor(t, o, 64);
    if (lane == 0) rstd_lds[lds_row0 + i * row_step] = 1.0f / sqrtf(t / (float)a.K + a.eps);
  }
}

template <bool WHOLE, bool P1>
__global__ __launch_bounds__(256) void gemm_wide_kernel(GemmArgs a, WideArgs x) {
  extern __shared__ float lds_f[];
  u32x4* bl = (u32x4*)lds_f;                          // [2 stages][kWideFrags][64 lanes]
  float* rstd_lds = lds_f + 2 * kWideFrags * 64 * 4;  // [128]
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int wm = w & 1, wn = w >> 1;  // this wave: row tiles wm*4..+3, n-tiles wn*4..+3 of the group
  const int nrole = WHOLE ? 1 : a.W;
  const int cg = (int)blockIdx.x / nrole, role = (int)blockIdx.x % nrole;
  const int nsl = (WHOLE ? a.W : 1) * a.P;  // slices this workgroup walks
  constexpr int kStages = 16 / kWideStage;  // stages per slice (even: the LDS buffer of a stage is its parity)
  constexpr int nblk = kWideStage * 4;      // (k-step, row tile) blocks per stage

  const u32x4* wbase[4];
#pragma unroll
  for (int ra = 0; ra < 4; ++ra) {
    const int t = min(cg * kWideWgTiles + wn * 4 + ra, a.ntiles - 1);
    wbase[ra] = a.wp + lane + (size_t)t * a.kst * 64;
  }
  // first k-step of stage s of the j-th slice this workgroup walks
  auto kstep0 = [&](int j, int s) {
    const int wj = WHOLE ? j / a.P : role, p = WHOLE ? j % a.P : j;
    return (p * a.W + wj) * 16 + s * kWideStage;
  };
  // wave w stages k-step w of a stage: 16 fragments (row tile, half); ActPack fragments are already
  // in consumer lane order
  auto b_src = [&](int k0) { return a.actp + (size_t)(k0 + w) * (kWideRowTiles * 2 * 64) + lane; };
  u32x4 areg[2][4][kWideStage], breg[2 * kWideRowTiles];
  auto store_b = [&](int buf) {
    u32x4* dst = bl + ((size_t)buf * kWideFrags + w * (2 * kWideRowTiles)) * 64 + lane;
#pragma unroll
    for (int i = 0; i < 2 * kWideRowTiles; ++i) dst[i * 64] = breg[i];
  };

  // acc: the slice being accumulated; run: running sum of this role's slices (P > 1); tot: sum of
  // the finished roles (WHOLE)
  f32x4 acc[4][4], run[4][4], tot[4][4];
  const f32x4 zero = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int ra = 0; ra < 4; ++ra)
#pragma unroll
    for (int r = 0; r < 4; ++r) acc[ra][r] = run[ra][r] = tot[ra][r] = zero;

  {
    const int k0 = kstep0(0, 0);
#pragma unroll
    for (int ks = 0; ks < kWideStage; ++ks)
#pragma unroll
      for (int ra = 0; ra < 4; ++ra) areg[0][ra][ks] = wbase[ra][(size_t)(k0 + ks) * 64];
    const u32x4* src = b_src(k0);
#pragma unroll
    for (int i = 0; i < 2 * kWideRowTiles; ++i) breg[i] = src[i * 64];
  }
  if (WHOLE && a.ssq_in != nullptr) {
    wide_rstd_rows<16>(a, w, 4, lane, rstd_lds, w);
    wide_rstd_rows<16>(a, w + 64, 4, lane, rstd_lds, w + 64);
  }
  store_b(0);
  __syncthreads();

  for (int j = 0; j < nsl; ++j) {
#pragma unroll
    for (int s = 0; s < kStages; ++s) {
      // While stage s is multiplied out of LDS buffer s & 1 and areg[s & 1], the next stage is
      // requested, two loads per block so that the wave never sits in a long run of load issues:
      // first its activations (written to LDS at the end of this stage), then its weights.  After
      // the very last stage the workgroup's first stage is requested again (and never used).
      const bool last = s == kStages - 1 && j + 1 == nsl;
      const int k1 = last ? kstep0(0, 0) : (s == kStages - 1 ? kstep0(j + 1, 0) : kstep0(j, s + 1));
      const u32x4* src = b_src(k1);
      const u32x4* bp = bl + ((size_t)(s & 1) * kWideFrags + wm * 4 * 2) * 64 + lane;
      u32x4 bq[kWideAhead + 1][2];
      auto fetch = [&](int blk) {
        const int ks = blk >> 2, r = blk & 3;
        bq[blk % (kWideAhead + 1)][0] = bp[((ks * kWideRowTiles + r) * 2) * 64];
        bq[blk % (kWideAhead + 1)][1] = bp[((ks * kWideRowTiles + r) * 2 + 1) * 64];
      };
#pragma unroll
      for (int blk = 0; blk < kWideAhead; ++blk) fetch(blk);
#pragma unroll
      for (int blk = 0; blk < nblk; ++blk) {
        const int ks = blk >> 2, r = blk & 3;
        if (blk + kWideAhead < nblk) fetch(blk + kWideAhead);
        if (blk < nblk / 2) {
          breg[2 * blk] = src[(2 * blk) * 64];
          breg[2 * blk + 1] = src[(2 * blk + 1) * 64];
        } else {
#pragma unroll
          for (int q = (blk - nblk / 2) * 2; q < (blk - nblk / 2) * 2 + 2; ++q)
            areg[(s + 1) & 1][q & 3][q >> 2] = wbase[q & 3][(size_t)(k1 + (q >> 2)) * 64];
        }
        // (keeps the requests where they are written: spread over the blocks, LDS reads kWideAhead
        // blocks ahead of their use)
        __builtin_amdgcn_sched_barrier(0);
        const bf16x8 bh = as_bf16x8(bq[blk % (kWideAhead + 1)][0]), bo = as_bf16x8(bq[blk % (kWideAhead + 1)][1]);
        const bool first = s == 0 && ks == 0;  // a slice starts from zero
#pragma unroll
        for (int ra = 0; ra < 4; ++ra)
          acc[ra][r] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(areg[s & 1][ra][ks]), bh,
                                                               first ? zero : acc[ra][r], 0, 0, 0);
#pragma unroll
        for (int ra = 0; ra < 4; ++ra)
          acc[ra][r] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(areg[s & 1][ra][ks]), bo, acc[ra][r], 0, 0, 0);
      }
      store_b((s + 1) & 1);
      __syncthreads();
    }
    // the slice is complete: fold it into the role's running sum, a complete role into the total
    const int wj = WHOLE ? j / a.P : role, p = WHOLE ? j % a.P : j;
#pragma unroll
    for (int ra = 0; ra < 4; ++ra)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        if constexpr (P1) {
          if constexpr (WHOLE) tot[ra][r] = tot[ra][r] + acc[ra][r];  // (zero + first role)
        } else {
          run[ra][r] = p == 0 ? acc[ra][r] : run[ra][r] + acc[ra][r];
          if constexpr (WHOLE) {
            if (p == a.P - 1) tot[ra][r] = (wj == 0 ? zero : tot[ra][r]) + run[ra][r];
          }
        }
      }
  }

#pragma unroll
  for (int ra = 0; ra < 4; ++ra) {
    const int t = cg * kWideWgTiles + wn * 4 + ra;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int rt = wm * 4 + r;
      if (t < a.ntiles && rt < x.row_tiles) {
        if constexpr (WHOLE) {
          const int row = rt * 16 + (lane & 15);
          const float rstd = (a.ssq_in != nullptr && row < a.m) ? rstd_lds[row] : 1.0f;
          epilogue_quad<false>(a, t, row, lane, tot[ra][r], rstd, false, zero, zero);
        } else {
          x.partials[(((size_t)role * a.ntiles + t) * kWideRowTiles + rt) * 64 + lane] = P1 ? acc[ra][r] : run[ra][r];
        }
      }
    }
  }
}

// split mode, second half: add the W running sums of every 16 x 16 tile in the order w = 0..W-1 and
// finish it.  Workgroup (4 n-tiles, row tile), one tile per wave; all W sums are requested at once.
constexpr int kWideMaxRoles = 8;  // W <= 8 (launch shape)
__global__ __launch_bounds__(256) void gemm_wide_finish_kernel(GemmArgs a, WideArgs x) {
  __shared__ float rstd_lds[16];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int rt = (int)blockIdx.y;
  const int t = (int)blockIdx.x * 4 + w;
  const bool norm = a.ssq_in != nullptr;
  const f32x4 zero = f32x4{0.f, 0.f, 0.f, 0.f};
  f32x4 pv[kWideMaxRoles];
#pragma unroll
  for (int ww = 0; ww < kWideMaxRoles; ++ww)
    if (ww < a.W && t < a.ntiles) pv[ww] = x.partials[(((size_t)ww * a.ntiles + t) * kWideRowTiles + rt) * 64 + lane];
  if (norm) wide_rstd_rows<4>(a, rt * 16 + w * 4, 1, lane, rstd_lds, w * 4);
  __syncthreads();
  if (t >= a.ntiles) return;
  const int row = rt * 16 + (lane & 15);
  const float rstd = (norm && row < a.m) ? rstd_lds[lane & 15] : 1.0f;
  f32x4 v = zero;
#pragma unroll
  for (int ww = 0; ww < kWideMaxRoles; ++ww)
    if (ww < a.W) v += pv[ww];
  epilogue_quad<false>(a, t, row, lane, v, rstd, false, zero, zero);
}

// whole mode when the column groups alone give every compute unit most of a workgroup
static bool wide_whole(int ntiles, int n_cu) {
  const int ncg = (ntiles + kWideWgTiles - 1) / kWideWgTiles;
  return ncg * 4 >= n_cu * 3;
}

// Measured on the 8B shapes at 116 rows: products whose columns fill the device (gate/up, LM head)
// and K-split ones with at least ~100 MB of weights (down) are faster here; for the smaller ones
// (QKV, O) the second kernel of the split costs more than the narrow kernel's L2 re-reads.
bool gemm_wide_preferred(int N, int K) {
  const int n_cu = device_cu_count();
  const long ntiles = (N + 15) / 16;
  return n_cu > 0 && (wide_whole((int)ntiles, n_cu) || ntiles * (K / 32) >= 100000);
}

size_t gemm_wide_workspace_bytes(int N, int K) {
  const int n_cu = device_cu_count();
  const int ntiles = (N + 15) / 16;
  if (n_cu <= 0 || wide_whole(ntiles, n_cu)) return 0;
  int W = 1;
  for (int cand = 8; cand >= 1; --cand)
    if ((K / 512) % cand == 0) { W = cand; break; }
  return (size_t)W * ntiles * kWideRowTiles * 64 * sizeof(f32x4);
}

template <bool WHOLE, bool P1>
static hipError_t launch_wide_variant(const GemmArgs& a, const WideArgs& x, int grid, bool timed, hipEvent_t e0,
                                      hipEvent_t e1, hipStream_t st) {
  static bool attr_set = false;  // more than 64 KB of dynamic LDS has to be allowed once per kernel
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)gemm_wide_kernel<WHOLE, P1>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)kWideLdsBytes);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  // whole mode: the kernel's own start and end are the GEMM's; split mode: start of the first
  // kernel, end of the second
  if (timed)
    hipExtLaunchKernelGGL((gemm_wide_kernel<WHOLE, P1>), dim3(grid), dim3(256), (uint32_t)kWideLdsBytes, st, e0,
                          WHOLE ? e1 : nullptr, 0, a, x);
  else
    gemm_wide_kernel<WHOLE, P1><<<grid, 256, kWideLdsBytes, st>>>(a, x);
  return hipGetLastError();
}

hipError_t launch_gemm_wide(const GemmCall& c, GemmArgs a, hipStream_t st) {
  const int n_cu = device_cu_count();
  if (c.act_tiles != kWideRowTiles || a.K % 512 != 0 || a.W > kWideMaxRoles) return hipErrorInvalidValue;
  WideArgs x{};
  x.ncg = (a.ntiles + kWideWgTiles - 1) / kWideWgTiles;
  x.row_tiles = (c.m + 15) / 16;
  const bool whole = wide_whole(a.ntiles, n_cu);
  const bool timed = c.ev_start != nullptr && c.ev_stop != nullptr;
  hipError_t e;
  if (whole) {
    e = a.P == 1 ? launch_wide_variant<true, true>(a, x, x.ncg, timed, c.ev_start, c.ev_stop, st)
                 : launch_wide_variant<true, false>(a, x, x.ncg, timed, c.ev_start, c.ev_stop, st);
    return e;
  }
  const size_t need = (size_t)a.W * a.ntiles * kWideRowTiles * 64 * sizeof(f32x4);
  if (c.wide_ws == nullptr || c.wide_ws_bytes < need) return hipErrorInvalidValue;
  x.partials = (f32x4*)c.wide_ws;
  e = a.P == 1 ? launch_wide_variant<false, true>(a, x, x.ncg * a.W, timed, c.ev_start, c.ev_stop, st)
               : launch_wide_variant<false, false>(a, x, x.ncg * a.W, timed, c.ev_start, c.ev_stop, st);
  if (e != hipSuccess) return e;
  const dim3 fgrid((a.ntiles + 3) / 4, x.row_tiles);
  if (timed)
    hipExtLaunchKernelGGL(gemm_wide_finish_kernel, fgrid, dim3(256), 0, st, nullptr, c.ev_stop, 0, a, x);
  else
    gemm_wide_finish_kernel<<<fgrid, 256, 0, st>>>(a, x);
  return hipGetLastError();
}

}  // namespace pipesd
