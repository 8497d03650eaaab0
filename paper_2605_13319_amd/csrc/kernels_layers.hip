// All decoder layers of a NAV pass in ONE cooperative kernel (bf16 models, passes of up to 16 rows).
//
// Launching one kernel per projection costs ~6 us of launch gap, pipeline ramp and tail for each of
// the ~160 dependent steps of a pass, during which HBM idles.  Here one workgroup per compute unit
// stays resident for the whole layer stack and the steps are separated by a device-wide barrier
// instead.  What that buys: every wave requests the first weight chunk of the next projection
// BEFORE it enters the barrier (weights depend on nothing), so the HBM stream keeps running while
// the workgroups synchronise and while the small activation tensors make their way across.
//
// Cross-workgroup traffic (ActPack buffers, residual stream, queries, new cache rows, attention
// partials, sums of squares) is written through to memory (sc1 stores, see device_gemm.h) and lives
// in per-layer buffers that are written once per pass (ActArena), so readers use ordinary cached
// loads and the barrier needs no cache write-back or invalidate: measured on MI355X, 2.3 us per
// barrier against 14-17 us with fences and ~2.5 us for a kernel boundary.
//
// The barrier is a monotone counter per group of workgroups plus one top counter; a waiter gives up
// after a bounded number of polls, raises an error flag and every workgroup leaves the kernel, so a
// lost workgroup can never hang the device.
#include "device_attn.h"

namespace pipesd {

struct LayersArgs {
  LayerSlabs sl;
  const float* final_norm;
  int n_layers;
  GemmArgs gemm[4];  // QKV, O, gate/up, down; per-layer fields (weights, buffers, gains) are filled in on the device
  ActArena arena;
  int nsplit, head_dim;
  unsigned long long* step_clock;  // optional [4 * n_layers + 1]
  unsigned* bar;  // [0]: top counter; [32 * (1 + g)]: counter of group g = workgroup % 8; zeroed before launch
  int* err;       // set to 1 if a barrier timed out
};

constexpr unsigned kBarGroups = 8;
constexpr unsigned kBarMaxPolls = 2000000u;  // x ~0.1-0.2 us per poll: a fraction of a second

// Workgroup barrier without memory fences: in-flight (hand-issued) weight loads must stay in flight.
__device__ __forceinline__ void wg_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Device-wide barrier in two halves, so that work which does not depend on other workgroups (the
// request for the next projection's first weights) can sit between "I am done" and "is everybody
// done".  grid_arrive: every wave has drained its stores (Xwg<true>::drain) before calling.
// grid_wait returns false (to every thread of the workgroup) if it timed out or another workgroup
// reported an error.
__device__ __forceinline__ void grid_arrive(unsigned* bar, unsigned& gen) {
  ++gen;
  wg_barrier();
  if (threadIdx.x == 0) {
    const unsigned grp = blockIdx.x % kBarGroups, per = gridDim.x / kBarGroups;
    unsigned* gc = bar + 32 * (1 + grp);
    const unsigned prev = __hip_atomic_fetch_add(gc, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (prev == gen * per - 1u) __hip_atomic_fetch_add(bar, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}
__device__ __forceinline__ bool grid_wait(unsigned* bar, int* err, unsigned gen, int* fail_lds) {
  if (threadIdx.x == 0) {
    int fail = 0;
    unsigned polls = 0;
    while (__hip_atomic_load(bar, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < gen * kBarGroups) {
      __builtin_amdgcn_s_sleep(1);
      if ((++polls & 1023u) == 0u) {
        if (polls > kBarMaxPolls || __hip_atomic_load(err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) {
          __hip_atomic_store(err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          fail = 1;
          break;
        }
      }
    }
    *fail_lds = fail;
  }
  wg_barrier();
  return *fail_lds == 0;
}
__device__ __forceinline__ bool grid_sync(unsigned* bar, int* err, unsigned& gen, int* fail_lds) {
  grid_arrive(bar, gen);
  return grid_wait(bar, err, gen, fail_lds);
}

__device__ __forceinline__ TeamPos team_pos(const GemmArgs& g, int w) {
  const int tpw = 8 / g.W;  // teams per workgroup (8 waves)
  TeamPos tp;
  tp.tl = w / g.W;
  tp.wt = w % g.W;
  tp.active = w < tpw * g.W;
  tp.team = (int)blockIdx.x * tpw + tp.tl;
  tp.nteams = (int)gridDim.x * tpw;
  return tp;
}

// per-layer fields of GEMM `ph` (0 QKV, 1 O, 2 gate/up, 3 down) of layer l
__device__ __forceinline__ void patch_layer(GemmArgs& g, const LayersArgs& a, int l, int ph) {
  const LayerSlabs& sl = a.sl;
  const ActArena& ar = a.arena;
  g.layer = l;
  if (ph == 0) {
    g.wp = (const u32x4*)(sl.wqkv + l * sl.qkv_bytes);
    g.actp = (const u32x4*)ar.xa(l);
    g.ssq_in = ar.sa(l);
    if (l > 0) g.ssq_parts = a.gemm[1].ntiles;  // after the first layer the sums of squares come per n-tile
    g.out = ar.q(l);
  } else if (ph == 1) {
    g.wp = (const u32x4*)(sl.wo + l * sl.o_bytes);
    g.actp = (const u32x4*)ar.ap(l);
    g.res_in = ar.ra(l);
    g.out = ar.rb(l);
    g.outp = (u32x4*)ar.xb(l);
    g.ssq_out = ar.sb(l);
    g.gain_next = (const float*)(sl.ffn_norm + l * sl.norm_bytes);
  } else if (ph == 2) {
    g.wp = (const u32x4*)(sl.wgu + l * sl.gu_bytes);
    g.actp = (const u32x4*)ar.xb(l);
    g.ssq_in = ar.sb(l);
    g.outp = (u32x4*)ar.gp(l);
  } else {
    g.wp = (const u32x4*)(sl.wdown + l * sl.down_bytes);
    g.actp = (const u32x4*)ar.gp(l);
    g.res_in = ar.rb(l);
    g.out = ar.ra(l + 1);
    g.outp = (u32x4*)ar.xa(l + 1);
    g.ssq_out = ar.sa(l + 1);
    g.gain_next = l + 1 < a.n_layers ? (const float*)(sl.attn_norm + (l + 1) * sl.norm_bytes) : a.final_norm;
  }
}

template <int HD>
__global__ __launch_bounds__(512) void layers_kernel(LayersArgs a) {
  extern __shared__ float lds[];
  __shared__ int fail_lds;
  constexpr int KS = 16;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  unsigned gen = 0;
  u32x4 af[KS];
  {
    GemmArgs g = a.gemm[0];
    patch_layer(g, a, 0, 0);
    gemm_prefetch<KS>(g, team_pos(g, w), lane, af);
  }
  const int nsteps = 4 * a.n_layers;
  for (int step = 0; step < nsteps; ++step) {
    const int l = step >> 2, ph = step & 3;
    if (a.step_clock != nullptr && blockIdx.x == 0 && tid == 0) a.step_clock[step] = wall_clock64();
    {
      GemmArgs g = a.gemm[ph];
      patch_layer(g, a, l, ph);
      gemm_body<1, KS, true>(g, team_pos(g, w), 8 / g.W, 8, lds, af);
    }
    Xwg<true>::drain();
    if (ph == 0) {
      // attention over the paged cache: tasks (kv head, 256-token split), then the split merge
      const GemmArgs& gq = a.gemm[0];
      if (!grid_sync(a.bar, a.err, gen, &fail_lds)) return;
      const int nkv = gq.kv.n_kv_heads, nqt = (gq.n_q_heads / nkv * gq.m + 15) / 16;
      const int ntasks = nkv * a.nsplit * nqt;
      for (int task = blockIdx.x; task < ntasks; task += gridDim.x) {
        attn_task<HD, true>(a.arena.q(l), gq.kv, l, gq.m, gq.start_pos, gq.n_q_heads, a.nsplit, a.arena.partials(l),
                            task % nkv, (task / nkv) % a.nsplit, task / (nkv * a.nsplit), task / (nkv * a.nsplit) + 1,
                            lds);
        __syncthreads();  // the task's LDS is free again
      }
      Xwg<true>::drain();
      if (!grid_sync(a.bar, a.err, gen, &fail_lds)) return;
      const int nmerge = gq.m * gq.n_q_heads * (HD / 8);
      for (int gt = blockIdx.x * 512 + tid; gt < nmerge; gt += gridDim.x * 512)
        attn_merge_thread<true>(a.arena.partials(l), gq.m, gq.n_q_heads, HD, a.nsplit, (u32x4*)a.arena.ap(l), gt);
      Xwg<true>::drain();
    }
    if (step + 1 < nsteps) {
      // the next projection's first weights are requested before the barrier: they depend on nothing
      grid_arrive(a.bar, gen);
      GemmArgs g = a.gemm[(step + 1) & 3];
      patch_layer(g, a, (step + 1) >> 2, (step + 1) & 3);
      gemm_prefetch<KS>(g, team_pos(g, w), lane, af);
      if (!grid_wait(a.bar, a.err, gen, &fail_lds)) return;
    }
  }
  if (a.step_clock != nullptr && blockIdx.x == 0 && tid == 0) a.step_clock[nsteps] = wall_clock64();
}

// ------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------
int device_cu_count();

size_t act_arena_layout(ActArena& a, int n_layers, int d_model, int q_dim, int d_ffn, bool per_layer, int act_tiles) {
  const size_t L = per_layer ? (size_t)n_layers : 0, R = (size_t)act_tiles * 16;
  a.x_bytes = act_pack_bytes(d_model, act_tiles);
  a.ap_bytes = act_pack_bytes(q_dim, act_tiles);
  a.gp_bytes = act_pack_bytes(d_ffn, act_tiles);
  a.r_bytes = R * d_model * sizeof(float);
  a.q_bytes = R * q_dim * sizeof(float);
  a.ssq_stride = d_model / 16;
  a.s_bytes = (R * a.ssq_stride * sizeof(float) + 255) / 256 * 256;
  size_t off = 0;
  a.off_xa = off; off += (L + 1) * a.x_bytes;
  a.off_xb = off; off += L * a.x_bytes;
  a.off_ap = off; off += L * a.ap_bytes;
  a.off_gp = off; off += L * a.gp_bytes;
  a.off_ra = off; off += (L + 1) * a.r_bytes;
  a.off_rb = off; off += L * a.r_bytes;
  a.off_q = off; off += L * a.q_bytes;
  a.off_sa = off; off += (L + 1) * a.s_bytes;
  a.off_sb = off; off += L * a.s_bytes;
  if (!per_layer) {  // one buffer of each kind: every layer's accessor lands on it
    off = 0;
    a.off_xa = off; off += a.x_bytes;
    a.off_xb = off; off += a.x_bytes;
    a.off_ap = off; off += a.ap_bytes;
    a.off_gp = off; off += a.gp_bytes;
    a.off_ra = off; off += a.r_bytes;
    a.off_rb = off; off += a.r_bytes;
    a.off_q = off; off += a.q_bytes;
    a.off_sa = off; off += a.s_bytes;
    a.off_sb = off; off += a.s_bytes;
    a.x_bytes = a.ap_bytes = a.gp_bytes = a.r_bytes = a.q_bytes = a.s_bytes = 0;
  }
  return off;
}

static bool team_shape(int N, int K, int grid, GemmArgs& g) {
  if (K % 512 != 0) return false;
  const int slices = K / 512;
  int W = 1;
  for (int cand = 8; cand >= 1; --cand)
    if (slices % cand == 0) { W = cand; break; }
  g.K = K;
  g.N = N;
  g.ntiles = (N + 15) / 16;
  g.kst = K / 32;
  g.W = W;
  g.P = slices / W;
  const int tpw = 8 / W, nteams = grid * tpw;
  const int tmax = 56 / (tpw * W);  // LDS reduce area of the workgroup stays under 56 KB
  int best_tg = 1;
  long best_cost = -1;
  for (int tg = 1; tg <= tmax; ++tg) {
    const int groups = (g.ntiles + tg - 1) / tg;
    const long rounds = (groups + nteams - 1) / nteams;
    const long cost = rounds * tg;
    if (best_cost < 0 || cost <= best_cost) { best_cost = cost; best_tg = tg; }
  }
  g.tg = best_tg;
  return true;
}

bool layers_fused_supported(const LayersCall& c) {
  const int n_cu = device_cu_count();
  if (n_cu < 8 || n_cu % 8 != 0) return false;
  if (c.m < 1 || c.m > 16) return false;
  if (c.head_dim != 64 && c.head_dim != 128) return false;
  if (c.d_model % 512 || c.q_dim % 512 || c.d_ffn % 512) return false;
  if (c.d_model / 16 > 256) return false;  // sums of squares per row are fetched 4 per lane
  return true;
}

hipError_t launch_layers(const LayersCall& c, hipStream_t st) {
  if (!layers_fused_supported(c)) return hipErrorInvalidValue;
  const int grid = device_cu_count();
  LayersArgs a{};
  a.sl = c.slabs;
  a.final_norm = c.final_norm;
  a.n_layers = c.n_layers;
  a.arena = c.arena;
  a.step_clock = c.step_clock;
  a.nsplit = (c.start_pos + c.m + kAttnWgTokens - 1) / kAttnWgTokens;
  a.head_dim = c.head_dim;
  a.bar = c.bar;
  a.err = (int*)(c.bar + (1 + kBarGroups) * 32);
  const int nqkv = c.q_dim + 2 * c.kv.n_kv_heads * c.head_dim;
  GemmArgs base{};
  base.row_tiles = 1;
  base.act_tiles = 2;
  base.m = c.m;
  base.eps = c.eps;
  base.ssq_stride = c.arena.ssq_stride;
  base.rope_cs = c.rope_cs;
  base.kv = c.kv;
  base.start_pos = c.start_pos;
  base.n_q_heads = c.n_q_heads;
  a.gemm[0] = base;
  if (!team_shape(nqkv, c.d_model, grid, a.gemm[0])) return hipErrorInvalidValue;
  a.gemm[0].ssq_parts = 1;  // the row setup leaves one sum per row
  a.gemm[0].epi = EPI_QKV;
  a.gemm[0].ldo = c.q_dim;
  a.gemm[1] = base;
  if (!team_shape(c.d_model, c.q_dim, grid, a.gemm[1])) return hipErrorInvalidValue;
  a.gemm[1].epi = EPI_RESID;
  a.gemm[1].ldo = c.d_model;
  a.gemm[2] = base;
  if (!team_shape(2 * c.d_ffn, c.d_model, grid, a.gemm[2])) return hipErrorInvalidValue;
  a.gemm[2].ssq_parts = c.d_model / 16;
  a.gemm[2].epi = EPI_SWIGLU;
  a.gemm[3] = base;
  if (!team_shape(c.d_model, c.d_ffn, grid, a.gemm[3])) return hipErrorInvalidValue;
  a.gemm[3].epi = EPI_RESID;
  a.gemm[3].ldo = c.d_model;

  size_t lds_floats = attn_lds_floats(c.head_dim);
  for (const GemmArgs* g : {&a.gemm[0], &a.gemm[1], &a.gemm[2], &a.gemm[3]}) {
    const size_t f = gemm_lds_floats(g->tg, g->W, 1, 8 / g->W);
    if (f > lds_floats) lds_floats = f;
  }
  size_t lds = lds_floats * sizeof(float);
  hipError_t e = hipMemsetAsync(c.bar, 0, (1 + kBarGroups) * 32 * sizeof(unsigned), st);  // counters; the flag is sticky
  if (e != hipSuccess) return e;
  void* args[] = {&a};
  static bool lds_allowed = false;  // more than 64 KB of dynamic LDS has to be asked for once per kernel
  if (!lds_allowed) {
    const int cap = (int)(attn_lds_floats(128) * sizeof(float)) > 64 * 1024 ? (int)(attn_lds_floats(128) * sizeof(float)) : 64 * 1024;
    e = hipFuncSetAttribute((const void*)layers_kernel<128>, hipFuncAttributeMaxDynamicSharedMemorySize, cap);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void*)layers_kernel<64>, hipFuncAttributeMaxDynamicSharedMemorySize, cap);
    if (e != hipSuccess) return e;
    lds_allowed = true;
  }
  if (c.head_dim == 128)
    return hipLaunchCooperativeKernel((const void*)layers_kernel<128>, dim3(grid), dim3(512), args, lds, st);
  return hipLaunchCooperativeKernel((const void*)layers_kernel<64>, dim3(grid), dim3(512), args, lds, st);
}

}  // namespace pipesd
