// Router of the MoE layer on one GPU (paper Section 3.2 and Alg. 3 with |G| = 1):
// per-expert loads, even split of every expert's assignments over its vExperts, bucket
// offsets, and the slot of every assignment in the per-vExpert contiguous layout
// (Section 4, expert-wise layout transformation).
//
// Integer-only and deterministic: ranks are stable in assignment id, obtained from
// per-wave LDS histograms, a prefix over the waves' histograms, and ballot-based ranks
// inside a wave -- never from the arrival order of atomics.
//
// The assignments are cut into `units` of unit_len consecutive ids; one wavefront owns one
// unit.  Kernel 1 writes hist[unit][e].  Kernel 2: every block re-derives, for its own four
// units, the number of earlier assignments per expert (prefix over units), the replica
// shares and bucket offsets, then places its assignments.
// Up to 4096 assignments the whole router is one workgroup of sixteen waves instead
// (route_fused_kernel): the same steps with the histograms kept in LDS and every wave's
// assignments held in registers, one launch instead of two.
#include "common.h"

namespace flexmoe {

constexpr int kRouteThreads = 256;
constexpr int kRouteWaves = kRouteThreads / kWave;

int route_units(int A, int* unit_len) {
  int len = A <= 65536 ? 256 : 512;     // short units: the placement rounds of a unit run one after another
  if ((A + len - 1) / len > 1024) len = (int)align_up((size_t)(A + 1023) / 1024, 64);
  *unit_len = len;
  int u = (A + len - 1) / len;
  return u < 1 ? 1 : u;
}

size_t route_ws_bytes(int A, int E) {
  int len;
  return align_up((size_t)route_units(A, &len) * E * sizeof(int32_t), 256);
}


// Even split of expert e's `tot` assignments over its replicas (Section 3.2): floor share q, the
// first m = tot mod n_e replicas in list order take one more.  Fills the per-vExpert share and
// the rank (within the expert) at which each vExpert's chunk starts.
__device__ __forceinline__ void split_expert(int e, int tot, const uint16_t* roff, const uint16_t* rids, int32_t* eq,
                                             int32_t* em, int32_t* vcount, int32_t* vstart,
                                             int32_t* __restrict__ vexpert_owner, bool write_owner) {
  const int o = roff[e], n = roff[e + 1] - o;
  const int q = tot / n, m = tot - q * n;
  eq[e] = q;
  em[e] = m;
  for (int r = 0; r < n; ++r) {
    const int v = rids[o + r];
    vcount[v] = q + (r < m ? 1 : 0);
    vstart[v] = r * q + min(r, m);
    if (write_owner) vexpert_owner[v] = e;
  }
}

// Places the 64 assignments base_a .. base_a+63 of one wave (lane's expert id e, -1 = none).
// Stable rank = assignments of the same expert before this wave's unit (wbase_w[e], advanced as
// the rounds go by) + same-expert lanes below this one (ballot match over the 9-bit key).
__device__ __forceinline__ void place_round(int a, int e, int lane, int32_t* wbase_w, const int32_t* eq,
                                            const int32_t* em, const uint16_t* roff, const uint16_t* rids,
                                            const int32_t* voff, const int32_t* vstart, int32_t* __restrict__ dest,
                                            int32_t* __restrict__ src) {
  const unsigned long long lt = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  const unsigned key = (e < 0) ? 0x100u : (unsigned)e;   // 9 bits
  unsigned long long peers = ~0ull;
#pragma unroll
  for (int b = 0; b < 9; ++b) {
    const bool bit = (key >> b) & 1u;
    const unsigned long long bal = __ballot(bit);
    peers &= bit ? bal : ~bal;
  }
  if (e >= 0) {
    const int before = __popcll(peers & lt);
    const int rank = wbase_w[e] + before;
    if (before == 0) wbase_w[e] += __popcll(peers);   // the group's lowest lane advances the count
    const int q = eq[e], m = em[e];
    const int cut = m * (q + 1);
    const int r = (rank < cut) ? rank / (q + 1) : m + (rank - cut) / q;
    const int v = rids[roff[e] + r];
    const int p = voff[v] + rank - vstart[v];
    dest[a] = p;
    src[p] = a;
  }
}

__global__ __launch_bounds__(kRouteThreads) void route_hist_kernel(const int32_t* __restrict__ idx, int A, int E,
                                                                   int units, int unit_len,
                                                                   int32_t* __restrict__ hist) {
  __shared__ int32_t h[kRouteWaves][FLEXMOE_MAX_EXPERTS];
  const int w = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const int u = blockIdx.x * kRouteWaves + w;
  for (int e = lane; e < E; e += kWave) h[w][e] = 0;
  __syncthreads();
  if (u < units) {
    const int lo = u * unit_len;
    const int hi = min(lo + unit_len, A);
    for (int a = lo + lane; a < hi; a += kWave) {
      int e = idx[a];
      if ((unsigned)e < (unsigned)E) atomicAdd(&h[w][e], 1);
    }
  }
  __syncthreads();
  if (u < units)
    for (int e = lane; e < E; e += kWave) hist[(size_t)u * E + e] = h[w][e];
}

template <typename Tab>
__global__ __launch_bounds__(kRouteThreads) void route_assign_kernel(
    const int32_t* __restrict__ idx, int A, int E, int V, int units, int unit_len, Tab tab,
    const int32_t* __restrict__ hist, int32_t* __restrict__ expert_count, int32_t* __restrict__ vexpert_count,
    int32_t* __restrict__ vexpert_off, int32_t* __restrict__ vexpert_owner, int32_t* __restrict__ dest,
    int32_t* __restrict__ src) {
  __shared__ int32_t part_tot[kRouteThreads], part_pre[kRouteThreads];
  __shared__ int32_t wbase[kRouteWaves][FLEXMOE_MAX_EXPERTS];
  __shared__ int32_t eq[FLEXMOE_MAX_EXPERTS], em[FLEXMOE_MAX_EXPERTS];
  __shared__ uint16_t roff[FLEXMOE_MAX_EXPERTS + 1], rids[FLEXMOE_MAX_VEXPERTS];
  __shared__ int32_t vcount[FLEXMOE_MAX_VEXPERTS], vstart[FLEXMOE_MAX_VEXPERTS], voff[FLEXMOE_MAX_VEXPERTS + 1];
  __shared__ int32_t scan[kRouteThreads];

  const int tid = threadIdx.x;
  const int w = tid / kWave, lane = tid % kWave;
  const int u0 = blockIdx.x * kRouteWaves;

  for (int i = tid; i <= E; i += kRouteThreads) roff[i] = tab.rep_off[i];
  for (int i = tid; i < V; i += kRouteThreads) rids[i] = tab.rep_ids[i];

  // loads per expert over all units, and over the units before this block's first one
  int ep = 1;
  while (ep < E) ep <<= 1;
  const int parts = kRouteThreads / ep;
  {
    const int e = tid & (ep - 1), part = tid / ep;
    int tot = 0, pre = 0;
    if (e < E)
      for (int u = part; u < units; u += parts) {
        int c = hist[(size_t)u * E + e];
        tot += c;
        if (u < u0) pre += c;
        else if (u < u0 + kRouteWaves) wbase[u - u0][e] = c;     // this block's own units: kept for the wave bases
      }
    part_tot[tid] = tot;
    part_pre[tid] = pre;
  }
  __syncthreads();
  if (tid < E) {
    const int e = tid;
    int tot = 0, pre = 0;
    for (int p = 0; p < parts; ++p) {
      tot += part_tot[p * ep + e];
      pre += part_pre[p * ep + e];
    }
    int run = pre;
    for (int ww = 0; ww < kRouteWaves; ++ww) {
      const int own = (u0 + ww < units) ? wbase[ww][e] : 0;       // histogram of unit u0 + ww, left there above
      wbase[ww][e] = run;
      run += own;
    }
    split_expert(e, tot, roff, rids, eq, em, vcount, vstart, vexpert_owner, blockIdx.x == 0);
    if (blockIdx.x == 0) expert_count[e] = tot;
  }
  __syncthreads();

  // exclusive prefix sum of vcount in ascending vExpert id (two entries per thread)
  {
    const int a0 = (2 * tid < V) ? vcount[2 * tid] : 0;
    const int a1 = (2 * tid + 1 < V) ? vcount[2 * tid + 1] : 0;
    // inclusive scan inside each wave by shuffles, then the waves' totals through LDS
    int incl = a0 + a1;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
      const int up = __shfl_up(incl, o);
      if (lane >= o) incl += up;
    }
    if (lane == kWave - 1) scan[w] = incl;
    __syncthreads();
    int before = 0;
#pragma unroll
    for (int ww = 0; ww < kRouteWaves; ++ww)
      if (ww < w) before += scan[ww];
    const int excl = before + incl - (a0 + a1);
    if (2 * tid < V) voff[2 * tid] = excl;
    if (2 * tid + 1 < V) voff[2 * tid + 1] = excl + a0;
    if (tid == kRouteThreads - 1) voff[V] = before + incl;   // == A for valid input
  }
  __syncthreads();
  if (blockIdx.x == 0) {
    for (int v = tid; v < V; v += kRouteThreads) {
      vexpert_count[v] = vcount[v];
      vexpert_off[v] = voff[v];
    }
    if (tid == 0) vexpert_off[V] = voff[V];
  }

  // place this wave's unit: stable rank = earlier units + earlier rounds + lower lanes
  const int u = u0 + w;
  if (u >= units) return;
  const int lo = u * unit_len;
  const int hi = min(lo + unit_len, A);
  // the expert id of the next round is fetched while the current round is placed
  auto fetch = [&](int base_a) {
    const int a = base_a + lane;
    int e = -1;
    if (a < hi) {
      e = idx[a];
      if ((unsigned)e >= (unsigned)E) e = -1;
    }
    return e;
  };
  int e_next = fetch(lo);
  for (int base_a = lo; base_a < hi; base_a += kWave) {
    const int e = e_next;
    e_next = fetch(base_a + kWave);
    place_round(base_a + lane, e, lane, wbase[w], eq, em, roff, rids, voff, vstart, dest, src);
  }
}

// ---------------------------------------------------------------------------------------------
// The whole router in one workgroup (A <= kFusedMaxA): wave w owns the assignments
// [w*unit_len, (w+1)*unit_len), at most 4 per lane, loaded once into registers.
// ---------------------------------------------------------------------------------------------
constexpr int kFusedThreads = 1024;
constexpr int kFusedWaves = kFusedThreads / kWave;
constexpr int kFusedRounds = 4;
constexpr int kFusedMaxA = kFusedWaves * kWave * kFusedRounds;

template <typename Tab>
__global__ __launch_bounds__(kFusedThreads) void route_fused_kernel(
    const int32_t* __restrict__ idx, int A, int E, int V, Tab tab, int32_t* __restrict__ expert_count,
    int32_t* __restrict__ vexpert_count, int32_t* __restrict__ vexpert_off, int32_t* __restrict__ vexpert_owner,
    int32_t* __restrict__ dest, int32_t* __restrict__ src) {
  __shared__ int32_t wbase[kFusedWaves][FLEXMOE_MAX_EXPERTS];       // histograms, then prefixes over waves
  __shared__ int32_t eq[FLEXMOE_MAX_EXPERTS], em[FLEXMOE_MAX_EXPERTS];
  __shared__ uint16_t roff[FLEXMOE_MAX_EXPERTS + 1], rids[FLEXMOE_MAX_VEXPERTS];
  __shared__ int32_t vcount[FLEXMOE_MAX_VEXPERTS], vstart[FLEXMOE_MAX_VEXPERTS], voff[FLEXMOE_MAX_VEXPERTS + 1];
  __shared__ int32_t wave_tot[FLEXMOE_MAX_VEXPERTS / kWave];

  const int tid = threadIdx.x;
  const int w = tid / kWave, lane = tid % kWave;
  const int unit_len = ((A + kFusedWaves - 1) / kFusedWaves + kWave - 1) / kWave * kWave;
  const int rounds = unit_len / kWave;                               // <= kFusedRounds (host check)
  const int lo = w * unit_len, hi = min(lo + unit_len, A);

  int ev[kFusedRounds];
#pragma unroll
  for (int r = 0; r < kFusedRounds; ++r) {
    const int a = lo + r * kWave + lane;
    ev[r] = -1;
    if (r < rounds && a < hi) ev[r] = idx[a];
  }
  for (int i = tid; i <= E; i += kFusedThreads) roff[i] = tab.rep_off[i];
  for (int i = tid; i < V; i += kFusedThreads) rids[i] = tab.rep_ids[i];
  for (int i = tid; i < kFusedWaves * FLEXMOE_MAX_EXPERTS; i += kFusedThreads) (&wbase[0][0])[i] = 0;
  __syncthreads();
#pragma unroll
  for (int r = 0; r < kFusedRounds; ++r) {
    if ((unsigned)ev[r] >= (unsigned)E) ev[r] = -1;
    if (r < rounds && ev[r] >= 0) atomicAdd(&wbase[w][ev[r]], 1);
  }
  __syncthreads();
  if (tid < E) {
    const int e = tid;
    int run = 0;
    for (int ww = 0; ww < kFusedWaves; ++ww) {
      const int c = wbase[ww][e];
      wbase[ww][e] = run;
      run += c;
    }
    split_expert(e, run, roff, rids, eq, em, vcount, vstart, vexpert_owner, true);
    expert_count[e] = run;
  }
  __syncthreads();
  // exclusive prefix sum of vcount in ascending vExpert id: one entry per thread, wave scans + wave totals
  {
    const int c = (tid < V) ? vcount[tid] : 0;
    int incl = c;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
      const int up = __shfl_up(incl, o);
      if (lane >= o) incl += up;
    }
    if (tid < FLEXMOE_MAX_VEXPERTS && lane == kWave - 1) wave_tot[w] = incl;
    __syncthreads();
    if (tid < FLEXMOE_MAX_VEXPERTS) {
      int before = 0;
      for (int ww = 0; ww < w; ++ww) before += wave_tot[ww];
      if (tid < V) {
        voff[tid] = before + incl - c;
        vexpert_count[tid] = c;
        vexpert_off[tid] = before + incl - c;
      }
      if (tid == V - 1) {
        voff[V] = before + incl;             // == A for valid input
        vexpert_off[V] = before + incl;
      }
    }
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < kFusedRounds; ++r)
    if (r < rounds && lo + r * kWave < hi)
      place_round(lo + r * kWave + lane, ev[r], lane, wbase[w], eq, em, roff, rids, voff, vstart, dest, src);
}

template <typename Tab>
static hipError_t launch_route_t(const int32_t* idx, int A, int E, int V, const Tab& tab, int32_t* expert_count,
                                 int32_t* vexpert_count, int32_t* vexpert_off, int32_t* vexpert_owner, int32_t* dest,
                                 int32_t* src, void* ws, hipStream_t s) {
  if (A <= kFusedMaxA) {
    hipLaunchKernelGGL(route_fused_kernel<Tab>, dim3(1), dim3(kFusedThreads), 0, s, idx, A, E, V, tab, expert_count,
                       vexpert_count, vexpert_off, vexpert_owner, dest, src);
    return hipGetLastError();
  }
  int unit_len;
  const int units = route_units(A, &unit_len);
  const int blocks = (units + kRouteWaves - 1) / kRouteWaves;
  int32_t* hist = (int32_t*)ws;
  hipLaunchKernelGGL(route_hist_kernel, dim3(blocks), dim3(kRouteThreads), 0, s, idx, A, E, units, unit_len, hist);
  hipLaunchKernelGGL(route_assign_kernel<Tab>, dim3(blocks), dim3(kRouteThreads), 0, s, idx, A, E, V, units, unit_len,
                     tab, hist, expert_count, vexpert_count, vexpert_off, vexpert_owner, dest, src);
  return hipGetLastError();
}

hipError_t launch_route(const int32_t* idx, int A, int E, int V, const PlacementArg& tab, int32_t* expert_count,
                        int32_t* vexpert_count, int32_t* vexpert_off, int32_t* vexpert_owner, int32_t* dest,
                        int32_t* src, void* ws, hipStream_t s) {
  if (E <= PlacementArgSmall::kMaxExperts && V <= PlacementArgSmall::kMaxVexperts) {
    PlacementArgSmall small;
    for (int e = 0; e <= E; ++e) small.rep_off[e] = tab.rep_off[e];
    for (int e = E + 1; e <= PlacementArgSmall::kMaxExperts; ++e) small.rep_off[e] = 0;
    for (int v = 0; v < PlacementArgSmall::kMaxVexperts; ++v) small.rep_ids[v] = v < V ? tab.rep_ids[v] : 0;
    return launch_route_t(idx, A, E, V, small, expert_count, vexpert_count, vexpert_off, vexpert_owner, dest, src, ws, s);
  }
  return launch_route_t(idx, A, E, V, tab, expert_count, vexpert_count, vexpert_off, vexpert_owner, dest, src, ws, s);
}

}  // namespace flexmoe
