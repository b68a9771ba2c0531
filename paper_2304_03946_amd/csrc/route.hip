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
#include "common.h"

namespace flexmoe {

constexpr int kRouteThreads = 256;
constexpr int kRouteWaves = kRouteThreads / kWave;

int route_units(int A, int* unit_len) {
  int len = 512;
  if ((A + len - 1) / len > 1024) len = (int)align_up((size_t)(A + 1023) / 1024, 64);
  *unit_len = len;
  int u = (A + len - 1) / len;
  return u < 1 ? 1 : u;
}

size_t route_ws_bytes(int A, int E) {
  int len;
  return align_up((size_t)route_units(A, &len) * E * sizeof(int32_t), 256);
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

__global__ __launch_bounds__(kRouteThreads) void route_assign_kernel(
    const int32_t* __restrict__ idx, int A, int E, int V, int units, int unit_len, PlacementArg tab,
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
      wbase[ww][e] = run;
      if (u0 + ww < units) run += hist[(size_t)(u0 + ww) * E + e];
    }
    // even split over the n_e replicas: floor share q, the first m replicas take one more
    const int o = roff[e], n = roff[e + 1] - o;
    const int q = tot / n, m = tot - q * n;
    eq[e] = q;
    em[e] = m;
    for (int r = 0; r < n; ++r) {
      const int v = rids[o + r];
      vcount[v] = q + (r < m ? 1 : 0);
      vstart[v] = r * q + min(r, m);
      if (blockIdx.x == 0) vexpert_owner[v] = e;
    }
    if (blockIdx.x == 0) expert_count[e] = tot;
  }
  __syncthreads();

  // exclusive prefix sum of vcount in ascending vExpert id (two entries per thread)
  {
    const int a0 = (2 * tid < V) ? vcount[2 * tid] : 0;
    const int a1 = (2 * tid + 1 < V) ? vcount[2 * tid + 1] : 0;
    scan[tid] = a0 + a1;
    __syncthreads();
    for (int s = 1; s < kRouteThreads; s <<= 1) {
      int add = (tid >= s) ? scan[tid - s] : 0;
      __syncthreads();
      scan[tid] += add;
      __syncthreads();
    }
    const int excl = scan[tid] - (a0 + a1);
    if (2 * tid < V) voff[2 * tid] = excl;
    if (2 * tid + 1 < V) voff[2 * tid + 1] = excl + a0;
    if (tid == kRouteThreads - 1) voff[V] = scan[tid];   // == A for valid input
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
  const unsigned long long lt = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  for (int base_a = lo; base_a < hi; base_a += kWave) {
    const int a = base_a + lane;
    int e = -1;
    if (a < hi) {
      e = idx[a];
      if ((unsigned)e >= (unsigned)E) e = -1;
    }
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
      const int rank = wbase[w][e] + before;
      if (before == 0) wbase[w][e] += __popcll(peers);   // the group's lowest lane advances the count
      const int q = eq[e], m = em[e];
      const int cut = m * (q + 1);
      const int r = (rank < cut) ? rank / (q + 1) : m + (rank - cut) / q;
      const int v = rids[roff[e] + r];
      const int p = voff[v] + rank - vstart[v];
      dest[a] = p;
      src[p] = a;
    }
  }
}

hipError_t launch_route(const int32_t* idx, int A, int E, int V, const PlacementArg& tab, int32_t* expert_count,
                        int32_t* vexpert_count, int32_t* vexpert_off, int32_t* vexpert_owner, int32_t* dest,
                        int32_t* src, void* ws, hipStream_t s) {
  int unit_len;
  const int units = route_units(A, &unit_len);
  const int blocks = (units + kRouteWaves - 1) / kRouteWaves;
  int32_t* hist = (int32_t*)ws;
  hipLaunchKernelGGL(route_hist_kernel, dim3(blocks), dim3(kRouteThreads), 0, s, idx, A, E, units, unit_len, hist);
  hipLaunchKernelGGL(route_assign_kernel, dim3(blocks), dim3(kRouteThreads), 0, s, idx, A, E, V, units, unit_len,
                     tab, hist, expert_count, vexpert_count, vexpert_off, vexpert_owner, dest, src);
  return hipGetLastError();
}

}  // namespace flexmoe
