// GEMM for passes of 65..256 rows (batched verification of many clients, prompt ingestion).
//
// At this many rows the activations of a K slice no longer fit a wave's registers, and spreading the
// rows over workgroups that re-read the weights from the L2 (the narrow kernel's way) moves many
// times the weights through it.  Here a workgroup of sixteen or eight waves (four or two per SIMD)
// multiplies ALL rows of the pass with 8 n-tiles of weights.  Both operands reach the matrix cores through LDS, and they
// get there without passing through registers: every wave asks for its share of a stage's fragments
// (per k-step the 8 weight fragments and the row tiles' activation fragments, hi and lo) with loads
// that write straight into LDS, into a ring of three (or four) stage buffers, two (three) stages
// ahead of the multiplies.  ActPack and the re-tiled weights are already in the lane order the
// matrix cores consume, so a fragment is 64 lanes x 16 bytes, copied as it is.  Per stage: wait until this wave's
// loads of the stage have landed (they return in order: all but the later stages' may be
// outstanding) and its own LDS reads have returned, one workgroup barrier, request the stage a
// ring's length minus one ahead into the buffer the barrier has just freed.  The multiplies run as
// a stream of blocks (k-step, row tile) whose operands are read from LDS one or three blocks ahead,
// across stage boundaries.  Wave (wm, wn) owns row tiles wm, wm + (waves / 2), .. x n-tiles
// wn*4 .. +3; row tiles past the pass are neither read nor multiplied.  Up to 128 rows the packed activations have 8 row tiles and a stage is two k-steps;
// up to 256 rows they have 16 and a stage is one (up to 192 rows only 12 of them are staged, and
// the ring has four buffers).
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

#include <type_traits>

#include "device_dma.h"
#include "device_gemm.h"

namespace pipesd {

// Shapes: ROWT = 8 row tiles (passes of 65..128 rows; the packed activations have 8 row tiles) with
// stages of two k-steps, and ROWT = 16 (129..256 rows; 16 row tiles) with stages of one.  Of the 16
// row tiles only the first RTL are brought into LDS: RTL = 12 for passes of up to 192 rows, whose
// smaller stages leave room for a fourth stage buffer (requests three stages ahead), else 16.
constexpr int wide_ring(int rtl) { return rtl == 12 ? 4 : 3; }  // stage buffers
constexpr int kWideWgTiles = 8;     // n-tiles per workgroup: 2 wave columns x 4
constexpr int wide_stage_ksteps(int rowt) { return rowt == 16 ? 1 : 2; }
// 1 KB fragments of one k-step in a stage buffer: the 8 weight fragments, then (row tile, half)
constexpr int wide_kstep_frags(int rowt) { return kWideWgTiles + 2 * rowt; }
constexpr size_t wide_ring_bytes(int rowt, int rtl) { return (size_t)wide_ring(rtl) * wide_stage_ksteps(rowt) * wide_kstep_frags(rtl) * 1024; }
constexpr size_t wide_max(size_t a, size_t b) { return a > b ? a : b; }
constexpr size_t kWideLdsBytes = wide_max(wide_ring_bytes(8, 8), wide_max(wide_ring_bytes(16, 12), wide_ring_bytes(16, 16))) + 256 * sizeof(float);

struct WideArgs {
  f32x4* partials;  // split: [W][ntiles][ROWT][64] running sums of role w
  int ncg;          // column groups of kWideWgTiles n-tiles
  int row_tiles;    // live row tiles of the pass
  int rowt;         // 8 or 16: row tiles of the packed activations (and of the partials)
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

// f(integral_constant<int, n>) for the run-time n in 0..N
template <int N, class F>
__device__ __forceinline__ void wide_dispatch_count(int n, F& f) {
  if constexpr (N == 0) {
    f(std::integral_constant<int, 0>{});
  } else {
    if (n == N) f(std::integral_constant<int, N>{});
    else wide_dispatch_count<N - 1>(n, f);
  }
}

// At least two waves per SIMD (one wave alone issues a matrix-core instruction only every ~30
// cycles): sixteen waves of one row tile each for 8 row tiles, eight waves of three or four row
// tiles each for 12 or 16.  Wave (wm, wn) = (w / 2, w % 2) owns row tiles r * (waves / 2) + wm x
// n-tiles wn*4 .. +3 of the group; waves w and w + 4 share a SIMD, so the live row tiles of a pass
// that does not fill its last tiles spread evenly over the SIMDs.
constexpr int wide_waves(int rowt) { return rowt == 8 ? 16 : 8; }
template <bool WHOLE, bool P1, int ROWT, int RTL>
__global__ __launch_bounds__(wide_waves(ROWT) * 64) void gemm_wide_kernel(GemmArgs a, WideArgs x) {
  extern __shared__ float lds_f[];
  constexpr int kWideWaves = wide_waves(ROWT), WMS = kWideWaves / 2;  // waves, wave rows
  constexpr int kWideRing = wide_ring(RTL);           // stage buffers
  constexpr int kWideStage = wide_stage_ksteps(ROWT); // k-steps per ring stage
  constexpr int kWideSliceStages = 16 / kWideStage;   // stages per 512-column slice
  constexpr int KF = wide_kstep_frags(RTL);           // fragments per k-step
  constexpr int SF = kWideStage * KF;                 // fragments per stage buffer
  constexpr int NPER = kWideStage * (kWideWgTiles + 2 * RTL) / kWideWaves;  // fragments this wave requests per stage
  constexpr int RW = RTL / WMS;                       // row tiles per wave
  u32x4* bl = (u32x4*)lds_f;                          // [kWideRing][SF][64 lanes]
  float* rstd_lds = lds_f + (kWideLdsBytes - 256 * sizeof(float)) / sizeof(float);  // [ROWT * 16]
  const int lane = threadIdx.x & 63, w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = w >> 1, wn = w & 1;  // row tiles r * WMS + wm, n-tiles wn*4 .. +3
  const int nrole = WHOLE ? 1 : a.W;
  const int cg = (int)blockIdx.x / nrole, role = (int)blockIdx.x % nrole;
  const int nsl = (WHOLE ? a.W : 1) * a.P;  // slices this workgroup walks

  // A stage's fragments, numbered f = ks * KF + (0..7 weights | 8.. activations (row tile, half)), are
  // dealt to the waves round robin: wave w requests f = w, w + kWideWaves, ..  What a wave asks for is
  // fixed for the whole walk except for the k-step, so each of its NPER requests keeps a source
  // pointer that moves on by one stage with every request (and by the jump to the next slice of the
  // walk at a slice boundary): no per-request index arithmetic on the scalar unit, which all waves of
  // the compute unit share.
  const char* rp[NPER];  // this lane's 16 bytes of fragment i of the next stage to request
  int rstep[NPER];       // bytes per k-step of that operand (wave-uniform)
  int rlds[NPER];        // where the fragment goes in a stage buffer (bytes)
  const int kslice0 = WHOLE ? 0 : role;  // first slice of the walk
#pragma unroll
  for (int i = 0; i < NPER; ++i) {
    const int f = w + kWideWaves * i, ks = f / KF, e = f % KF;  // (w is uniform)
    rlds[i] = f * 1024;
    if (e < kWideWgTiles) {
      rstep[i] = 1024;
      rp[i] = (const char*)(a.wp + ((size_t)min(cg * kWideWgTiles + e, a.ntiles - 1) * a.kst + ks) * 64 + lane);
    } else {  // ActPack is in consumer lane order
      rstep[i] = ROWT * 2 * 1024;
      rp[i] = (const char*)(a.actp + ((size_t)ks * (ROWT * 2) + (e - kWideWgTiles)) * 64 + lane);
    }
    rp[i] += (ptrdiff_t)(kslice0 * 16) * rstep[i];
  }
  // request this wave's share of the next stage into the stage buffer at byte offset `buf`
  auto request = [&](int buf) {
#pragma unroll
    for (int i = 0; i < NPER; ++i) {
      lds_dma16(rp[i], (char*)bl + buf + rlds[i]);
      rp[i] += (size_t)(kWideStage * rstep[i]);
    }
  };
  // the requests have covered a slice: move to the next slice of the walk (slice p*W + w follows
  // (p-1)*W + w; role w + 1 follows role w); past the end of the walk, to the last slice again
  int rq_j = 0, rq_p = 0;
  auto request_turn = [&]() {
    int dsl = 0;  // slices from the one just requested to the next
    if (rq_j + 1 < nsl) {
      dsl = a.W;
      if constexpr (WHOLE) {
        if (rq_p + 1 == a.P) dsl = 1 - (a.P - 1) * a.W;
      }
    }
    ++rq_j;
    rq_p = rq_p + 1 == a.P ? 0 : rq_p + 1;
    const int dk = (dsl - 1) * 16;  // (the pointers are already one slice further)
#pragma unroll
    for (int i = 0; i < NPER; ++i) rp[i] += (ptrdiff_t)(dk * rstep[i]);
  };

  // acc: the slice being accumulated; run: running sum of this role's slices (P > 1); tot: sum of
  // the finished roles (WHOLE)
  f32x4 acc[4][RW], run[4][RW], tot[4][RW];
  const f32x4 zero = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int ra = 0; ra < 4; ++ra)
#pragma unroll
    for (int r = 0; r < RW; ++r) acc[ra][r] = run[ra][r] = tot[ra][r] = zero;

  // The multiplies run as one stream of blocks (k-step, row tile of this wave): 8 MFMAs on a pair of
  // activation fragments (hi, lo) and the k-step's 4 weight fragments.  Operands are read from LDS
  // kAhead blocks ahead of their block.  When the block to read is the first of a stage, that stage
  // must have landed: this wave's loads of it have once at most the later stages' (ring - 2 of
  // them) are outstanding, and behind the workgroup barrier every wave's have.  The same wait covers
  // this wave's own LDS reads, so behind the barrier nobody reads the stage before any more, and
  // its buffer takes the stage ring - 1 ahead.  Past the end of the walk the last slice's first stages are requested and read
  // again (and never used), so the counts hold to the end.
  constexpr int BPS = kWideStage * RW;           // blocks per stage
  constexpr int kAhead = BPS >= 4 ? 3 : 1;       // (a power of two minus one, below BPS)
  constexpr int BPSL = kWideSliceStages * BPS;   // blocks per slice (a multiple of 4)
  constexpr int kStageBytes = SF * 1024;
  u32x4 bq[kAhead + 1][2];                       // ring of activation operand pairs
  constexpr int WR = RW >= kAhead ? 2 : 4;       // k-steps whose weight fragments are held (reads run at most that far ahead)
  u32x4 wfb[WR][4];                              // weight fragments of the last WR k-steps
  int rd = 0;                                    // stage buffer being read (byte offset in the ring)
  // this lane's 16 bytes of the wave's first weight fragment / first activation fragment in a stage buffer
  const char* lw = (const char*)bl + (wn * 4 * 64 + lane) * 16;
  const char* la = (const char*)bl + ((kWideWgTiles + wm * 2) * 64 + lane) * 16;
  // the next stage has landed for every wave and the stage before it is no longer read: move on to
  // it and ask for the stage ring - 1 ahead of it; s = the new stage's place in its slice
  auto stage_ready = [&](int s) {
    const int freed = rd;
    rd = rd == (kWideRing - 1) * kStageBytes ? 0 : rd + kStageBytes;
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(NPER * (kWideRing - 2)) : "memory");
    __builtin_amdgcn_s_barrier();
    if ((s + kWideRing - 1) % kWideSliceStages == 0) request_turn();
    request(freed);
  };

#pragma unroll
  for (int b = 0; b < kWideRing - 1; ++b) request(b * kStageBytes);
  if (WHOLE && a.ssq_in != nullptr) {
    constexpr int RPW = ROWT * 16 / kWideWaves;  // rows whose rstd this wave computes: w, w + kWideWaves, ..
#pragma unroll
    for (int h = 0; h < (RPW + 15) / 16; ++h)
      wide_rstd_rows<(RPW < 16 ? RPW : 16)>(a, w + 16 * kWideWaves * h, kWideWaves, lane, rstd_lds, w + 16 * kWideWaves * h);
  }
  asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(NPER * (kWideRing - 2)) : "memory");
  __builtin_amdgcn_s_barrier();
  request((kWideRing - 1) * kStageBytes);

  // The walk, compiled once per number LR of this wave's live row tiles (they are r*WMS + wm,
  // r < LR): a row tile past the pass is neither read nor multiplied, and no block asks whether it
  // is live.
  auto walk = [&](auto lrc) {
    constexpr int LR = decltype(lrc)::value;
    // read the operands of block b of the stage being read; kq = its k-step within the slice
    auto read_block = [&](int b, int kq, int slot) {
      const int ks = b / RW, r = b % RW;
      if (r == 0 && LR > 0) {
#pragma unroll
        for (int ra = 0; ra < 4; ++ra) wfb[kq & (WR - 1)][ra] = *(const u32x4*)(lw + rd + (ks * KF + ra) * 1024);
      }
      if (r < LR) {
        bq[slot][0] = *(const u32x4*)(la + rd + (ks * KF + r * WMS * 2) * 1024);
        bq[slot][1] = *(const u32x4*)(la + rd + (ks * KF + r * WMS * 2 + 1) * 1024);
      }
    };
#pragma unroll
    for (int b = 0; b < kAhead; ++b) read_block(b, b / RW, b);

    int p = 0, wj = kslice0;  // the slice being multiplied is p*W + wj
    for (int j = 0; j < nsl; ++j) {
#pragma unroll
      for (int bn = 0; bn < BPSL; ++bn) {
        {  // operands of the block kAhead ahead
          const int pn = (bn + kAhead) % BPSL;
          const int sn = pn / BPS, b = pn % BPS;
          if (b == 0) stage_ready(sn);
          read_block(b, pn / RW, pn & kAhead);
        }
        // (keeps the reads where they are written, kAhead blocks ahead of their use: left alone, the
        // scheduler sinks them to just in front of their multiplies and every block waits for LDS)
        __builtin_amdgcn_sched_barrier(0);
        const int kq = bn / RW, r = bn % RW;
        const bool first = kq == 0;  // a slice starts from zero
        if (r < LR) {
          const bf16x8 bh = as_bf16x8(bq[bn & kAhead][0]), bo = as_bf16x8(bq[bn & kAhead][1]);
#pragma unroll
          for (int ra = 0; ra < 4; ++ra)
            acc[ra][r] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(wfb[kq & (WR - 1)][ra]), bh, first ? zero : acc[ra][r], 0, 0, 0);
#pragma unroll
          for (int ra = 0; ra < 4; ++ra)
            acc[ra][r] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(wfb[kq & (WR - 1)][ra]), bo, acc[ra][r], 0, 0, 0);
        }
      }
      // The slice is complete: fold it into the role's running sum, a complete role into the total.
      // (The last products may have been issued in another basic block, where the compiler pads no
      // wait states for the adds below: spell them out.)
      __builtin_amdgcn_sched_barrier(0);
      asm volatile("s_nop 15\n\ts_nop 7" ::: "memory");
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int ra = 0; ra < 4; ++ra)
#pragma unroll
        for (int r = 0; r < LR; ++r) {
          if constexpr (P1) {
            if constexpr (WHOLE) tot[ra][r] = tot[ra][r] + acc[ra][r];  // (zero + first role)
          } else {
            run[ra][r] = p == 0 ? acc[ra][r] : run[ra][r] + acc[ra][r];
            if constexpr (WHOLE) {
              if (p == a.P - 1) tot[ra][r] = (wj == 0 ? zero : tot[ra][r]) + run[ra][r];
            }
          }
        }
      if (++p == a.P) {
        p = 0;
        if constexpr (WHOLE) ++wj;
      }
    }
  };
  {
    int lr = 0;  // this wave's live row tiles
#pragma unroll
    for (int r = 0; r < RW; ++r) lr += (r * WMS + wm < x.row_tiles) ? 1 : 0;
    wide_dispatch_count<RW>(lr, walk);
  }
  // the requests past the end of the walk must have landed before the workgroup gives its LDS back
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  if (WHOLE && a.ssq_in != nullptr) __syncthreads();  // (rstd_lds of the other waves)

#pragma unroll
  for (int ra = 0; ra < 4; ++ra) {
    const int t = cg * kWideWgTiles + wn * 4 + ra;
#pragma unroll
    for (int r = 0; r < RW; ++r) {
      const int rt = r * WMS + wm;
      if (t < a.ntiles && rt < x.row_tiles) {
        if constexpr (WHOLE) {
          const int row = rt * 16 + (lane & 15);
          const float rstd = (a.ssq_in != nullptr && row < a.m) ? rstd_lds[row] : 1.0f;
          epilogue_quad<false>(a, t, row, lane, tot[ra][r], rstd, false, zero, zero);
        } else {
          x.partials[(((size_t)role * a.ntiles + t) * ROWT + rt) * 64 + lane] = P1 ? acc[ra][r] : run[ra][r];
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
    if (ww < a.W && t < a.ntiles) pv[ww] = x.partials[(((size_t)ww * a.ntiles + t) * x.rowt + rt) * 64 + lane];
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
// Beyond 8 row tiles the narrow kernel's groups of up to 16 workgroups per weight stream lose more
// than the split's second launch costs: every product the wide kernel supports runs there.
bool gemm_wide_preferred(int N, int K, int row_tiles) {
  const int n_cu = device_cu_count();
  const long ntiles = (N + 15) / 16;
  return n_cu > 0 && (row_tiles > 8 || wide_whole((int)ntiles, n_cu) || ntiles * (K / 32) >= 100000);
}

size_t gemm_wide_workspace_bytes(int N, int K) {
  const int n_cu = device_cu_count();
  const int ntiles = (N + 15) / 16;
  if (n_cu <= 0 || wide_whole(ntiles, n_cu)) return 0;
  int W = 1;
  for (int cand = 8; cand >= 1; --cand)
    if ((K / 512) % cand == 0) { W = cand; break; }
  return (size_t)W * ntiles * 16 * 64 * sizeof(f32x4);  // (sized for the 16-row-tile shape)
}

template <bool WHOLE, bool P1, int ROWT, int RTL>
static hipError_t launch_wide_rowt(const GemmArgs& a, const WideArgs& x, int grid, bool timed, hipEvent_t e0,
                                   hipEvent_t e1, hipStream_t st) {
  static bool attr_set = false;  // more than 64 KB of dynamic LDS has to be allowed once per kernel
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)gemm_wide_kernel<WHOLE, P1, ROWT, RTL>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)kWideLdsBytes);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  // whole mode: the kernel's own start and end are the GEMM's; split mode: start of the first
  // kernel, end of the second
  const dim3 block(wide_waves(ROWT) * 64);
  if (timed)
    hipExtLaunchKernelGGL((gemm_wide_kernel<WHOLE, P1, ROWT, RTL>), dim3(grid), block, (uint32_t)kWideLdsBytes, st, e0,
                          WHOLE ? e1 : nullptr, 0, a, x);
  else
    gemm_wide_kernel<WHOLE, P1, ROWT, RTL><<<grid, block, kWideLdsBytes, st>>>(a, x);
  return hipGetLastError();
}

template <bool WHOLE, bool P1>
static hipError_t launch_wide_variant(const GemmArgs& a, const WideArgs& x, int grid, bool timed, hipEvent_t e0,
                                      hipEvent_t e1, hipStream_t st) {
  if (x.rowt == 16) {
    // (a whole-K walk with phases needs three accumulator sets of 64 registers: not built for 16 row tiles)
    if constexpr (WHOLE && !P1) return hipErrorInvalidValue;
    else if (x.row_tiles <= 12) return launch_wide_rowt<WHOLE, P1, 16, 12>(a, x, grid, timed, e0, e1, st);
    else return launch_wide_rowt<WHOLE, P1, 16, 16>(a, x, grid, timed, e0, e1, st);
  }
  return launch_wide_rowt<WHOLE, P1, 8, 8>(a, x, grid, timed, e0, e1, st);
}

// whether the wide kernel can run this product on `act_tiles` row tiles
bool gemm_wide_supported(int N, int K, int act_tiles) {
  if (act_tiles == 8) return true;
  if (act_tiles != 16) return false;
  const int n_cu = device_cu_count();
  const int ntiles = (N + 15) / 16;
  if (n_cu <= 0 || K % 512 != 0) return false;
  // the narrow kernel's split of K: W waves x P phases; whole-K walks need P == 1 here
  int W = 1;
  for (int cand = 8; cand >= 1; --cand)
    if ((K / 512) % cand == 0) { W = cand; break; }
  const int P = K / 512 / W;
  return !(wide_whole(ntiles, n_cu) && P != 1);
}

hipError_t launch_gemm_wide(const GemmCall& c, GemmArgs a, hipStream_t st) {
  const int n_cu = device_cu_count();
  if ((c.act_tiles != 8 && c.act_tiles != 16) || a.K % 512 != 0 || a.W > kWideMaxRoles) return hipErrorInvalidValue;
  WideArgs x{};
  x.ncg = (a.ntiles + kWideWgTiles - 1) / kWideWgTiles;
  x.row_tiles = (c.m + 15) / 16;
  x.rowt = c.act_tiles;
  const bool whole = wide_whole(a.ntiles, n_cu);
  const bool timed = c.ev_start != nullptr && c.ev_stop != nullptr;
  hipError_t e;
  if (whole) {
    e = a.P == 1 ? launch_wide_variant<true, true>(a, x, x.ncg, timed, c.ev_start, c.ev_stop, st)
                 : launch_wide_variant<true, false>(a, x, x.ncg, timed, c.ev_start, c.ev_stop, st);
    return e;
  }
  const size_t need = (size_t)a.W * a.ntiles * x.rowt * 64 * sizeof(f32x4);
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
