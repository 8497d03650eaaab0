// Device code of the skinny bf16 GEMM, shared by the per-GEMM kernel and the fused layer kernel.
//
// y[m][N] = act[m][K] * W[N][K]^T with few rows m (a client's k + 1 <= 32, or the rows of several
// clients, up to 128; the QKV / O / SwiGLU-FFN / LM-head products of the target forward, Sec. 2.2).  The pass is bound by streaming W once from HBM, so
// everything is arranged around that stream:
//  * W is re-tiled once, at model creation, into the order the matrix cores consume it: tile
//    (n-tile of 16 weight rows, k-step of 32 columns) is 1 KB, lane l holding row l%16, columns
//    8*(l/16)..+7.  A wave's load instruction then reads 1 KB contiguous and the data lands directly
//    in MFMA operand registers: no LDS pass, no barrier in the main loop.
//  * W is the A operand (16 weight rows x 32 k), the activations are the B operand (32 k x 16 rows).
//    Activations travel between kernels already in B-operand layout as a bf16 hi + lo pair (ActPack
//    in common.h): the producing epilogue splits each value once, every consuming wave just loads
//    registers.  Two MFMAs per weight fragment keep 16 significand bits of the activations; the
//    matrix cores idle otherwise.
//  * A pass of more than 16 rows is spread over GROUPS of workgroups that walk the same tiles, one
//    per 16 rows, placed on the same chiplet: the weights cross the memory interface once and the
//    other readers are served by the chiplet's L2.  (Beyond 64 rows the larger products go to the
//    kernel of kernels_gemm_wide.hip, which stages all rows' activations in LDS instead.)
//  * K is cut into W * P slices of KSTEPS*32 columns; a team of W waves takes slices p*W + w,
//    p = 0..P-1, one phase after the other, for a group of tg n-tiles, each wave keeping its running
//    16x16 sums in its own LDS slots; after the last phase the team adds them in a fixed order.
//    Nothing crosses teams: no global partials, no floating-point atomics; results are
//    bit-reproducible and independent of how groups are dealt to teams.
//  * RMSNorm is fused: the producer stores x * gain and per-tile sums of x^2; the consumer scales the
//    finished tile by rstd per row.
//  * Epilogues: plain store (logits), residual add (+ packed, gained copy for the next GEMM),
//    SiLU(gate)*up (packed), or rotary + query buffer / paged KV-cache append.  Rows 8..15 of a
//    weight tile are the partners of rows 0..7 (other half of the head for the rotary pair; the
//    up-projection row for a gate row) so a pair is finished inside one wave.
//
// CO ("coherent") selects how results are stored for other workgroups.  false: plain stores; the
// kernel boundary makes them visible.  true: inside one long-running kernel every such store is
// written through to memory (sc1) and drained before the device-wide barrier that orders it with
// its readers.  Loads are ordinary cached loads either way: the long-running kernel's buffers are
// single-assignment within a pass (ActArena), so no cache can hold an older copy of a line, and
// measured on MI355X a write-through store of part of a line never leaves stale neighbours behind
// in the writer's caches.  Weights, gains and rotary tables are immutable.
#pragma once

#include <type_traits>

#include "common.h"

namespace pipesd {

typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;

struct GemmArgs {
  const u32x4* wp;
  const u32x4* actp;      // packed activations (ActPack, K columns)
  const float* ssq_in;    // fused norm: [row][ssq_stride] partial sums of x^2, or nullptr
  int ssq_parts, ssq_stride;
  float* out;             // STORE: logits; RESID: new residual stream; QKV: query buffer (bf16 hi | lo halves per row)
  const float* res_in;    // RESID: residual stream the product is added to (may be `out`)
  u32x4* outp;            // RESID / SWIGLU: packed output for the next GEMM
  const float* gain_next; // RESID: gain applied to the packed copy
  float* ssq_out;         // RESID: [row][ssq_stride] per-tile sums of x_new^2
  const float* rope_cs;
  const RowMap* rows;     // QKV: per-row position and block table (several clients in the pass), or nullptr
  KvView kv;
  int m, K, N, ntiles, kst, W, P, tg, ldo, epi, layer, start_pos, n_q_heads;
  int row_tiles;          // workgroups that share a team's tiles, one per 16 rows of the pass (1..16)
  int act_tiles;          // row tiles of the pass's ActPack buffers
  float eps;
  const int32_t* gate;    // optional: the launch does nothing if this device word holds 0
};

// passes of at least this many row tiles take the wide kernel (kernels_gemm_wide.hip); `a` comes
// filled in by launch_gemm_bf16
constexpr int kWideMinRowTiles = 5;
hipError_t launch_gemm_wide(const GemmCall& c, GemmArgs a, hipStream_t st);
bool gemm_wide_preferred(int N, int K, int row_tiles);
bool gemm_wide_supported(int N, int K, int act_tiles);  // the wide kernel can run this product on ActPack buffers of that many row tiles

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// ---- hand-issued loads -------------------------------------------------------------------------
// The weight stream is issued and awaited by hand: the loads are opaque to the compiler's wait-count
// bookkeeping, and each use is preceded by an explicit s_waitcnt tied to the register it releases.
// Vector memory loads return in order, so "at most N younger loads outstanding" is exact; the
// compiler would otherwise join the with-next and without-next paths into vmcnt(0) and drain the
// pipeline at every chunk.  Stores are never issued by hand without trailing wait states: the
// hardware reads store data for a few cycles after issue and only the compiler tracks that.
// NT: non-temporal hint for weights that are read exactly once (a pass of up to 16 rows).  When two
// workgroups on the same chiplet read the same tiles (a pass of 17..32 rows) the loads are ordinary
// ones instead, so that the second reader finds the line in the L2.
template <bool NT>
__device__ __forceinline__ u32x4 stream_load(const u32x4* p) {
  u32x4 v;
  if constexpr (NT)
    asm volatile("global_load_dwordx4 %0, %1, off nt" : "=v"(v) : "v"(p));
  else
    asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(v) : "v"(p));
  return v;
}
__device__ __forceinline__ u32x4 act_load(const u32x4* p) {
  u32x4 v;
  asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(v) : "v"(p));
  return v;
}
constexpr int kSsqPerLane = 8;  // sums of squares per lane and row: up to 512 producer tiles (d_model <= 8192)

template <int N>
__device__ __forceinline__ void wait_younger(u32x4& v) {
  asm volatile("s_waitcnt vmcnt(%1)" : "+v"(v) : "n"(N));
}

// ---- stores of data other workgroups will read ---------------------------------------------------
template <bool CO>
struct Xwg {
  static __device__ __forceinline__ void st4(void* p, u32x4 v) {
    if constexpr (CO)
      asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 3" ::"v"(p), "v"(v) : "memory");
    else
      *(u32x4*)p = v;
  }
  static __device__ __forceinline__ void st4f(float* p, f32x4 v) { st4(p, __builtin_bit_cast(u32x4, v)); }
  static __device__ __forceinline__ void st2(void* p, u32x2 v) {
    if constexpr (CO)
      asm volatile("global_store_dwordx2 %0, %1, off sc1\n\ts_nop 3" ::"v"(p), "v"(v) : "memory");
    else
      *(u32x2*)p = v;
  }
  static __device__ __forceinline__ void st1(float* p, float v) {
    if constexpr (CO)
      asm volatile("global_store_dword %0, %1, off sc1\n\ts_nop 3" ::"v"(p), "v"(v) : "memory");
    else
      *p = v;
  }
  static __device__ __forceinline__ void st_u16(uint16_t* p, uint16_t v) {
    if constexpr (CO) {
      const unsigned w = v;
      asm volatile("global_store_short %0, %1, off sc1\n\ts_nop 3" ::"v"(p), "v"(w) : "memory");
    } else {
      *p = v;
    }
  }
  // all of this thread's stores have been acknowledged (call before signalling other workgroups)
  static __device__ __forceinline__ void drain() {
    if constexpr (CO) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  }
};

// split 8 consecutive columns k0..k0+7 (k0 % 8 == 0) of `row` into hi + lo and store them (ActPack)
template <bool CO>
__device__ __forceinline__ void store_act8x(u32x4* buf, int row, int k0, const float (&v)[8], int nt) {
  uint32_t h[4], l[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) split2_bf16(v[2 * i], v[2 * i + 1], h[i], l[i]);
  const int g = (k0 & 31) >> 3, c = row & 15;
  Xwg<CO>::st4(buf + act_index(k0 >> 5, row >> 4, 0, c, g, nt), u32x4{h[0], h[1], h[2], h[3]});
  Xwg<CO>::st4(buf + act_index(k0 >> 5, row >> 4, 1, c, g, nt), u32x4{l[0], l[1], l[2], l[3]});
}

// one chunk = KSTEPS weight fragments of one n-tile against this wave's activation fragments; while
// fragment ks is multiplied, fragment ks of the next chunk is requested into the same registers
template <int MT, int KSTEPS, bool NT, bool HAS_NEXT, int KS = 0>
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
    if constexpr (HAS_NEXT) af[KS] = stream_load<NT>(nxt + KS * 64);
    chunk_mfma<MT, KSTEPS, NT, HAS_NEXT, KS + 1>(af, bhi, blo, acc, nxt);
  } else {
    // The matrix cores deliver a product many cycles after issue and nothing but software keeps a
    // later reader of the accumulator away until then.  The compiler pads for that inside a basic
    // block, but the reader (the LDS store of the tile) may sit behind a block boundary where it was
    // seen to pad too little: the store then wrote what the registers held before.  So the padding
    // for the slowest product (16 passes: 19 wait states) is spelled out here, tied to the accumulators.
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) asm volatile("s_nop 15\n\ts_nop 7" : "+v"(acc[mt]));
  }
}

__device__ __forceinline__ f32x4 shfl4(f32x4 v, int src) {
  return f32x4{__shfl(v[0], src, 64), __shfl(v[1], src, 64), __shfl(v[2], src, 64), __shfl(v[3], src, 64)};
}

// Finish one n-tile with a whole wave: lane (gg = lane/16, cc = lane%16) holds the dot products of
// activation row `row` with weight rows gg*4 .. gg*4+3 of tile t.  Partner rows (i, i+8) sit 32 lanes
// apart and the two halves of an 8-column group 16 lanes apart, so pairs are joined by shuffles.
// Every lane of the wave must call this (rows beyond the pass only skip the stores).
// RESID: `pre` says that pre_res / pre_gain already hold this quad's residual and gain values.
// EPI: the epilogue as a compile-time constant (the per-projection kernels: only that epilogue's code
// and registers are in the kernel), or kEpiAny to pick by a.epi at run time (kernels that run several
// kinds of products).
constexpr int kEpiAny = -1;
template <bool CO, int EPI = kEpiAny>
__device__ __forceinline__ void epilogue_quad(const GemmArgs& a, int t, int row, int lane, f32x4 v, float rstd,
                                              bool pre, f32x4 pre_res, f32x4 pre_gain) {
  const int gg = lane >> 4;
  const bool live = row < a.m;
  switch (EPI == kEpiAny ? a.epi : EPI) {
    case EPI_STORE: {  // logits: read by later kernels only
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
      const size_t at = (size_t)row * a.ldo + t * 16 + gg * 4;
      f32x4 x = f32x4{0.f, 0.f, 0.f, 0.f};
      if (live) {
        x = (pre ? pre_res : *(const f32x4*)(a.res_in + at)) + v;
        Xwg<CO>::st4f(a.out + at, x);
      }
      float sq = x[0] * x[0] + x[1] * x[1] + x[2] * x[2] + x[3] * x[3];
      sq += __shfl_xor(sq, 16, 64);
      sq += __shfl_xor(sq, 32, 64);
      const f32x4 gn = pre ? pre_gain : *(const f32x4*)(a.gain_next + t * 16 + gg * 4);
      const f32x4 y = x * gn;
      const f32x4 hi4 = shfl4(y, lane + 16);  // columns +4..+7 of the 8-column group
      if (live && (gg & 1) == 0) {
        const float y8[8] = {y[0], y[1], y[2], y[3], hi4[0], hi4[1], hi4[2], hi4[3]};
        store_act8x<CO>(a.outp, row, t * 16 + gg * 4, y8, a.act_tiles);
        if (gg == 0) Xwg<CO>::st1(a.ssq_out + (size_t)row * a.ssq_stride + t, sq);
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
        store_act8x<CO>(a.outp, row, t * 8, y8, a.act_tiles);
      }
      break;
    }
    case EPI_QKV: {
      const f32x4 x1 = shfl4(v, lane + 32);
      if (!live || gg >= 2) break;
      const int h = a.kv.head_dim, half = h >> 1, hpt = h >> 4;
      const int hd = t / hpt, i0 = (t % hpt) * 8 + gg * 4;
      f32x4 r0, r1;
      if (hd < a.n_q_heads + a.kv.n_kv_heads) {
        const float* cs = a.rope_cs + ((size_t)row * half + i0) * 2;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float p0 = v[i] * rstd, p1 = x1[i] * rstd, c = cs[2 * i], sn = cs[2 * i + 1];
          r0[i] = p0 * c - p1 * sn;
          r1[i] = p1 * c + p0 * sn;
        }
      } else {
        r0 = v * rstd;
        r1 = x1 * rstd;
      }
      if (hd < a.n_q_heads) {
        // queries go to attention as the bf16 hi + lo pair its matrix-core operands are made of:
        // row = [ldo hi halves][ldo lo halves] (the bytes of ldo floats)
        uint16_t* o = (uint16_t*)(a.out + (size_t)row * a.ldo) + hd * h + i0;
        unsigned hh[2][2], ll[2][2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          const f32x4& rv = i == 0 ? r0 : r1;
          split2_bf16(rv[0], rv[1], hh[i][0], ll[i][0]);
          split2_bf16(rv[2], rv[3], hh[i][1], ll[i][1]);
        }
        Xwg<CO>::st2(o, u32x2{hh[0][0], hh[0][1]});
        Xwg<CO>::st2(o + half, u32x2{hh[1][0], hh[1][1]});
        Xwg<CO>::st2(o + a.ldo, u32x2{ll[0][0], ll[0][1]});
        Xwg<CO>::st2(o + a.ldo + half, u32x2{ll[1][0], ll[1][1]});
      } else {
        uint16_t* pool = (uint16_t*)a.kv.pool;
        KvView kvr = a.kv;  // the row's own client
        int pos = a.start_pos + row;
        if (a.rows != nullptr) {
          pos = a.rows->pos[row];
          kvr.table += a.rows->table_off[row];
        }
        const unsigned p0[2] = {pack2_bf16(r0[0], r0[1]), pack2_bf16(r0[2], r0[3])};
        const unsigned p1[2] = {pack2_bf16(r1[0], r1[1]), pack2_bf16(r1[2], r1[3])};
        if (hd < a.n_q_heads + a.kv.n_kv_heads) {
          const int kvh = hd - a.n_q_heads;
          Xwg<CO>::st2(pool + k_index(kvr, a.layer, pos, kvh, i0), u32x2{p0[0], p0[1]});
          Xwg<CO>::st2(pool + k_index(kvr, a.layer, pos, kvh, i0 + half), u32x2{p1[0], p1[1]});
        } else {
          const uint16_t b0[4] = {(uint16_t)p0[0], (uint16_t)(p0[0] >> 16), (uint16_t)p0[1], (uint16_t)(p0[1] >> 16)};
          const uint16_t b1[4] = {(uint16_t)p1[0], (uint16_t)(p1[0] >> 16), (uint16_t)p1[1], (uint16_t)(p1[1] >> 16)};
          const int kvh = hd - a.n_q_heads - a.kv.n_kv_heads;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            Xwg<CO>::st_u16(pool + v_index(kvr, a.layer, pos, kvh, i0 + i), b0[i]);
            Xwg<CO>::st_u16(pool + v_index(kvr, a.layer, pos, kvh, i0 + half + i), b1[i]);
          }
        }
      }
      break;
    }
  }
}

// A team = W consecutive waves of a workgroup.  `team` / `nteams` number the teams over the whole
// grid, `wt` is the wave's index in its team (waves with active == false belong to no team but must
// still take part in the workgroup barriers), `tl` the team's index inside the workgroup (selects
// its LDS area), `nwaves_wg` the workgroup's wave count.
// `row_base` (a multiple of 16) selects which 16 rows of the pass this team multiplies when the rows
// of a pass are spread over several workgroups (MT = 1 only).
struct TeamPos {
  int team, nteams, wt, tl;
  bool active;
  int row_base = 0;
};

template <int KSTEPS>
__device__ __forceinline__ const u32x4* gemm_chunk_ptr(const GemmArgs& a, int lane, int wt, int tile, int p) {
  return a.wp + lane + ((size_t)tile * a.kst + (size_t)(p * a.W + wt) * KSTEPS) * 64;
}

// request the first weight chunk of this wave (it does not depend on the activations, so it can be
// issued before whatever still separates the wave from the GEMM: a prologue, or a device-wide barrier)
template <int KSTEPS, bool NT = true>
__device__ __forceinline__ void gemm_prefetch(const GemmArgs& a, const TeamPos& tp, int lane, u32x4 (&af)[KSTEPS]) {
  const int ngroups = (a.ntiles + a.tg - 1) / a.tg;
  if (!tp.active || tp.team >= ngroups) return;
  const u32x4* first = gemm_chunk_ptr<KSTEPS>(a, lane, tp.wt, tp.team * a.tg, 0);
#pragma unroll
  for (int ks = 0; ks < KSTEPS; ++ks) af[ks] = stream_load<NT>(first + ks * 64);
}

// floats of LDS one workgroup needs: reduce slots of all its teams + rstd per row
__host__ __device__ inline size_t gemm_lds_floats(int tg, int W, int MT, int teams_per_wg) {
  return (size_t)teams_per_wg * tg * W * MT * 64 * 4 + 32;
}

// The GEMM proper.  All waves of the workgroup must call this together (it contains workgroup
// barriers).  EPI == kEpiAny (a kernel that runs several kinds of products): `af` must hold the
// in-flight first chunk (gemm_prefetch), the epilogue and the phase count are read from `a`.
// Otherwise (one kernel per kind of product) the body requests the first chunk itself, P1 says at
// compile time that a.P == 1, and the sums of squares are read iff the epilogue is not the residual one.
template <int MT, int KSTEPS, bool CO, bool NT = true, int EPI = kEpiAny, bool P1 = false>
__device__ __forceinline__ void gemm_body(const GemmArgs& a, const TeamPos& tp, int teams_per_wg, int nwaves_wg,
                                          float* lds, u32x4 (&af)[KSTEPS]) {
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  f32x4* red = (f32x4*)lds + (size_t)tp.tl * a.tg * a.W * MT * 64;        // [tg][W][MT][64]
  float* rstd_lds = lds + (size_t)teams_per_wg * a.tg * a.W * MT * 64 * 4;  // [MT*16]
  const int ngroups = (a.ntiles + a.tg - 1) / a.tg;
  const int iters = (ngroups + tp.nteams - 1) / tp.nteams;
  const int bc = lane & 15, bg = lane >> 4;

  // activation fragments of the current K slice (hi halves, then lo halves), awaited in full: they
  // and the first weight chunk are all needed before the first MFMA.  Lanes whose row is not part
  // of the pass load nothing: their MFMA columns are never stored.
  u32x4 bhi[MT][KSTEPS], blo[MT][KSTEPS];
  auto request_act = [&](int slice, int hl, u32x4 (&b)[MT][KSTEPS]) {
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
        if (tp.row_base + mt * 16 + bc < a.m)
          b[mt][ks] = act_load(a.actp + act_index(slice * KSTEPS + ks, mt + (tp.row_base >> 4), hl, bc, bg, a.act_tiles));
  };
  auto await_act = [&]() {
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        wait_younger<0>(bhi[mt][ks]);
        wait_younger<0>(blo[mt][ks]);
      }
  };
  // Fused norm: rstd per row from the producer's partial sums of squares, added in index order.  A
  // wave takes two rows at a time, up to kSsqPerLane partial sums per lane and row (the host checks
  // ssq_parts <= 64 * kSsqPerLane).  Everything the GEMM needs from the step before it is requested
  // in one go so that it arrives within one memory latency: the sums, the first quad's residual and
  // gain values (residual epilogue), the activation fragments.  Request and wait of the hand-issued
  // loads stay on one straight code path: a join of two paths would let the compiler copy registers
  // whose data is still on its way.
  const bool working = tp.active && tp.team < ngroups;
  const bool norm = a.ssq_in != nullptr;
  float part[2][kSsqPerLane];
  auto ssq_request = [&](int row0) {
#pragma unroll
    for (int r2 = 0; r2 < 2; ++r2)
#pragma unroll
      for (int j4 = 0; j4 < kSsqPerLane; ++j4) {
        const int row = row0 + r2 * nwaves_wg, j = lane + 64 * j4;
        part[r2][j4] = 0.f;
        // ("+v": the load lands in the very register that holds the zero of the lanes that skip it)
        if (norm && row < MT * 16 && tp.row_base + row < a.m && j < a.ssq_parts)
          asm volatile("global_load_dword %0, %1, off" : "+v"(part[r2][j4])
                       : "v"(a.ssq_in + (size_t)(tp.row_base + row) * a.ssq_stride + j));
      }
  };
  // `younger` = a constant number of hand-issued loads requested after the sums (they may stay in flight)
  auto ssq_finish = [&](int row0, auto younger) {
#pragma unroll
    for (int r2 = 0; r2 < 2; ++r2)
#pragma unroll
      for (int j4 = 0; j4 < kSsqPerLane; ++j4)
        asm volatile("s_waitcnt vmcnt(%1)" : "+v"(part[r2][j4]) : "n"(decltype(younger)::value));
#pragma unroll
    for (int r2 = 0; r2 < 2; ++r2) {
      const int row = row0 + r2 * nwaves_wg;
      float q = part[r2][0];
#pragma unroll
      for (int j4 = 1; j4 < kSsqPerLane; ++j4) q += part[r2][j4];
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) q += __shfl_xor(q, o, 64);
      if (norm && lane == 0 && row < MT * 16) rstd_lds[row] = 1.0f / sqrtf(q / (float)a.K + a.eps);
    }
  };
  // The same without a branch around the loads (the per-projection kernels): every lane loads, at
  // clamped indices, and the lanes without a partial sum of their own drop what they got after the
  // wait.  With a branch the value of the skipping lanes and the loaded value meet in a phi, and the
  // compiler is free to realise that phi by a copy right behind the load, of a register whose data
  // is still on its way (seen once; the ISA lint flags it).
  auto ssq_request_u = [&](int row0) {
#pragma unroll
    for (int r2 = 0; r2 < 2; ++r2)
#pragma unroll
      for (int j4 = 0; j4 < kSsqPerLane; ++j4) {
        const int row = min(tp.row_base + row0 + r2 * nwaves_wg, a.m - 1), j = min(lane + 64 * j4, a.ssq_parts - 1);
        asm volatile("global_load_dword %0, %1, off" : "=v"(part[r2][j4]) : "v"(a.ssq_in + (size_t)row * a.ssq_stride + j));
      }
  };
  auto ssq_finish_u = [&](int row0) {
#pragma unroll
    for (int r2 = 0; r2 < 2; ++r2)
#pragma unroll
      for (int j4 = 0; j4 < kSsqPerLane; ++j4) asm volatile("s_waitcnt vmcnt(0)" : "+v"(part[r2][j4]));
#pragma unroll
    for (int r2 = 0; r2 < 2; ++r2) {
      const int row = row0 + r2 * nwaves_wg;
      const bool live = row < MT * 16 && tp.row_base + row < a.m;
      float q = (live && lane < a.ssq_parts) ? part[r2][0] : 0.f;
#pragma unroll
      for (int j4 = 1; j4 < kSsqPerLane; ++j4) q += (live && lane + 64 * j4 < a.ssq_parts) ? part[r2][j4] : 0.f;
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) q += __shfl_xor(q, o, 64);
      if (lane == 0 && row < MT * 16) rstd_lds[row] = 1.0f / sqrtf(q / (float)a.K + a.eps);
    }
  };
  // residual epilogue: residual and gain values of the first quad this lane will finish
  f32x4 pre_res = f32x4{0.f, 0.f, 0.f, 0.f}, pre_gain = pre_res;
  bool have_pre = false;
  typedef std::integral_constant<int, 0> none_younger;
  if constexpr (EPI == kEpiAny) {
    // (ordinary loads: the compiler's own wait precedes whatever it does with the registers)
    if (working && a.epi == EPI_RESID) {
      const int t0 = tp.team * a.tg, e_first = tp.wt * 64 + lane;
      if (e_first < min(a.tg, a.ntiles - t0) * MT * 64) {
        const int tt = e_first / (MT * 64), rem = e_first % (MT * 64), l = rem & 63;
        const int row = tp.row_base + (rem >> 6) * 16 + (l & 15), col = (t0 + tt) * 16 + (l >> 4) * 4;
        if (row < a.m) pre_res = *(const f32x4*)(a.res_in + (size_t)row * a.ldo + col);
        pre_gain = *(const f32x4*)(a.gain_next + col);
        have_pre = true;
      }
    }
    ssq_request(w);
    if (working && a.P == 1) {
      request_act(tp.wt, 0, bhi);
      request_act(tp.wt, 1, blo);
      await_act();
    }
    ssq_finish(w, none_younger{});
    if (norm)
      for (int row0 = w + 2 * nwaves_wg; row0 < MT * 16; row0 += 2 * nwaves_wg) {
        ssq_request(row0);
        ssq_finish(row0, none_younger{});
      }
  } else {
    // The first weight chunk is requested first (the weights are the long pole and depend on
    // nothing), then what the step before left for this one (sums of squares, residual operands,
    // activation fragments), all without a wait in between, and then everything is awaited together.
    // (Awaiting the sums alone while the fragments are still in flight was tried: it gains nothing
    // measurable, and with the code between request and wait the compiler once moved a register whose
    // load was still on its way, which the ISA lint caught.)  A workgroup beyond the last tile group,
    // which only a padded grid has, requests the last group's chunk and never uses it.
    constexpr bool NORM = EPI != EPI_RESID;
    const int g0 = min(tp.team, ngroups - 1);
    {
      const u32x4* first = gemm_chunk_ptr<KSTEPS>(a, lane, tp.wt, g0 * a.tg, 0);
#pragma unroll
      for (int ks = 0; ks < KSTEPS; ++ks) af[ks] = stream_load<NT>(first + ks * 64);
    }
    if constexpr (NORM) ssq_request_u(w);
    if constexpr (EPI == EPI_RESID) {
      // unconditional loads at clamped indices: no branch, hence no join at which the compiler would
      // have to wait for them (a wait there would also drain the weight requests in front of them)
      const int t0 = g0 * a.tg, nq = min(a.tg, a.ntiles - t0) * MT * 64, e_first = tp.wt * 64 + lane;
      const int e = min(e_first, nq - 1);
      const int tt = e / (MT * 64), rem = e % (MT * 64), l = rem & 63;
      const int row = min(tp.row_base + (rem >> 6) * 16 + (l & 15), a.m - 1), col = (t0 + tt) * 16 + (l >> 4) * 4;
      pre_res = *(const f32x4*)(a.res_in + (size_t)row * a.ldo + col);
      pre_gain = *(const f32x4*)(a.gain_next + col);
      have_pre = working && e_first < nq;
    }
    if constexpr (P1) {
      request_act(tp.wt, 0, bhi);
      request_act(tp.wt, 1, blo);
    }
    if constexpr (P1) await_act();
    if constexpr (NORM) {
      ssq_finish_u(w);
      if (tp.row_base + 2 * nwaves_wg < a.m)  // (few waves and many rows: the remaining rows)
        for (int row0 = w + 2 * nwaves_wg; row0 < MT * 16; row0 += 2 * nwaves_wg) {
          ssq_request_u(row0);
          ssq_finish_u(row0);
        }
    }
  }
  for (int it = 0; it < iters; ++it) {
    const int grp = tp.team + it * tp.nteams;
    const bool on = tp.active && grp < ngroups;
    const int t0 = grp * a.tg;
    const int nt_g = on ? min(a.tg, a.ntiles - t0) : 0;
    const int e_first = tp.wt * 64 + lane;
    const bool pre = it == 0 && have_pre;
    if (on) {
      const int nphase = (EPI != kEpiAny && P1) ? 1 : a.P;
      for (int p = 0; p < nphase; ++p) {
        if ((EPI == kEpiAny || !P1) && a.P > 1) {
          request_act(p * a.W + tp.wt, 0, bhi);
          request_act(p * a.W + tp.wt, 1, blo);
          await_act();
        }
        for (int t = 0; t < nt_g; ++t) {
          const u32x4* nxt = nullptr;
          if (t + 1 < nt_g) nxt = gemm_chunk_ptr<KSTEPS>(a, lane, tp.wt, t0 + t + 1, p);
          else if (p + 1 < nphase) nxt = gemm_chunk_ptr<KSTEPS>(a, lane, tp.wt, t0, p + 1);
          else if (grp + tp.nteams < ngroups) nxt = gemm_chunk_ptr<KSTEPS>(a, lane, tp.wt, (grp + tp.nteams) * a.tg, 0);
          f32x4 acc[MT];
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
          if (nxt != nullptr)
            chunk_mfma<MT, KSTEPS, NT, true>(af, bhi, blo, acc, nxt);
          else
            chunk_mfma<MT, KSTEPS, NT, false>(af, bhi, blo, acc, nxt);
          // this wave's running sum over its phases lives in its own LDS slot
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) {
            f32x4* slot = red + ((size_t)(t * a.W + tp.wt) * MT + mt) * 64 + lane;
            *slot = (p == 0) ? acc[mt] : (*slot + acc[mt]);
          }
        }
      }
    }
    __syncthreads();
    // one lane per 4 tile rows x 1 activation row: add the W partial tiles, then finish with the wave
    if (on) {
      const int nquads = nt_g * MT * 64;
      for (int e = e_first; e < nquads; e += a.W * 64) {
        const int tt = e / (MT * 64), rem = e % (MT * 64), mt = rem >> 6, l = rem & 63;
        f32x4 v = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int ww = 0; ww < a.W; ++ww) v += red[((size_t)(tt * a.W + ww) * MT + mt) * 64 + l];
        const int lrow = mt * 16 + (l & 15), row = tp.row_base + lrow;
        const float rstd = (a.ssq_in != nullptr && row < a.m) ? rstd_lds[lrow] : 1.0f;
        epilogue_quad<CO, EPI>(a, t0 + tt, row, l, v, rstd, pre && e == e_first, pre_res, pre_gain);
      }
    }
    __syncthreads();  // red is free again
  }
}

}  // namespace pipesd
