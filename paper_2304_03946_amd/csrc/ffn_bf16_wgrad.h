// Weight-gradient kernels on the direct-to-LDS pipeline, the shared backward launch and the segment reduce.
// Part of the bf16 expert-FFN kernels; included by ffn_bf16.hip only (one translation unit).
#pragma once
#include "common.h"
#include "ffn_bf16_dma.h"
#include "ffn_bf16_persist.h"
namespace flexmoe {
// Work list of the weight-gradient kernels.  Experts are taken by descending load (ties by
// ascending id: the long contractions start first).  An expert's contraction runs over its
// non-empty buckets in ascending vExpert id, in K tiles of 32 tokens; with seg_tiles > 0 it is cut
// into segments of seg_tiles K tiles that different workgroups contract (a hot expert would
// otherwise be one long serial K loop): an expert with more than one segment leaves fp32 partial
// tiles in the workspace, `slot` numbering them, which wgrad_reduce_kernel adds up in segment
// order.  The whole list is a function of the bucket sizes only.  It is built once per backward call
// by wgrad_plan_kernel (one workgroup) and left in the workspace, where every workgroup of the two
// weight-gradient products finds its job with one load (deriving the list in each of the thousands of
// workgroups cost 4-5 us per output tile: 0.6 ms of the large layer's step).
struct WgradJob {
  int e;        // expert, -1: no job
  int seg;      // segment of the expert's contraction
  int nseg;     // segments of this expert
  int slot;     // index of the expert's first partial tile set (meaningful when nseg > 1)
};
// The work list exists twice, once per weight-gradient product, because the order of the jobs is also what spreads
// them over the XCDs: position j of the list owns grid rows j * m_tiles .. of the patched tile grid, whose patches
// go to the XCDs round-robin.  When a job's tiles fill fewer than eight patches (mid-size layers: two patches per
// job, or several jobs per patch), a list in descending load would hand the heaviest job of every round to the
// same XCDs (measured on the GPT-medium-like layer: two XCDs busy for 400 us, the others for 200-250).  So the jobs
// are dealt out heaviest first, each to the bin with the least work so far (balance_jobs; a bin = an XCD group, or,
// where several jobs share a patch, one of the patch's job slots: its workgroups are a fixed part of the XCD's
// compute units); a bin that holds a heavy job then gets fewer jobs, and the positions it leaves unused are holes
// (e = -1) that the kernels skip.
// `groups` and `per_slot` describe the product's geometry (wgrad_balance_geometry).
// Layout of the plan in the workspace (all int32 / int4, offsets in bytes from its 256-byte aligned start):
//   jobs      2 x [2 seg_rows_max] int4 {e, seg, nseg, slot} by list position (e = -1: no job): dW2's list, dW1's list
//   table     [FLEXMOE_MAX_EXPERTS] int4 {expert, segments, first slot, 0} by load rank (for wgrad_reduce_kernel)
//   boff      [E + 1]  int: expert e's non-empty buckets are entries boff[e] .. boff[e+1] of the two lists below
//   bstart    [V]      int: first row of the bucket
//   brows     [V]      int: rows of the bucket
//   etiles    [E]      int: 32-token K tiles of the expert (sum over its buckets of ceil(rows / 32))
//   njobs     [2]      int: positions of dW2's / dW1's list in use
struct WgradPlan {
  int4* jobs;             // the list of the product at hand (wgrad_plan_at's `product`: 0 = dW2, 1 = dW1)
  int4* jobs_other;
  int4* table;
  int* boff;
  int* bstart;
  int* brows;
  int* etiles;
  int* njobs;
};
__host__ __device__ inline size_t wgrad_plan_bytes(int seg_rows_max, int E, int V) {
  return (4 * (size_t)seg_rows_max + FLEXMOE_MAX_EXPERTS) * sizeof(int4) + (2 * (size_t)E + 4 + 2 * (size_t)V) * sizeof(int);
}
__host__ __device__ inline WgradPlan wgrad_plan_at(void* base, int seg_rows_max, int E, int V, int product = 0) {
  WgradPlan p;
  p.jobs = (int4*)base + (product ? 2 * seg_rows_max : 0);
  p.jobs_other = (int4*)base + (product ? 0 : 2 * seg_rows_max);
  p.table = (int4*)base + 4 * seg_rows_max;
  p.boff = (int*)(p.table + FLEXMOE_MAX_EXPERTS);
  p.bstart = p.boff + E + 1;
  p.brows = p.bstart + V;
  p.etiles = p.brows + V;
  p.njobs = p.etiles + E + (product ? 1 : 0);
  return p;
}

// How the positions of a product's work list map to XCDs: `groups` XCD groups take turns, `per_slot` consecutive
// jobs per turn.  groups = 1: nothing to balance (a job covers all XCDs evenly, or the geometry is irregular).
struct WgradBalance {
  int groups, per_slot;
};
__host__ __device__ inline WgradBalance wgrad_balance_geometry(int m_tiles, int n_tiles) {
  const int pw = patch_width(n_tiles), ph = kPatch / pw, npc = (n_tiles + pw - 1) / pw;
  if (pw * ph != kPatch) return WgradBalance{1, 1};
  if (m_tiles % ph == 0) {
    const int pj = (m_tiles / ph) * npc;                 // patches per job
    if (pj < kXcds && kXcds % pj == 0) return WgradBalance{kXcds / pj, 1};
    return WgradBalance{1, 1};
  }
  if (ph % m_tiles == 0 && npc == 1) return WgradBalance{kXcds, ph / m_tiles};      // several jobs per patch
  return WgradBalance{1, 1};
}
constexpr int kPlanJobsLds = 1024;      // work lists up to this length are balanced (longer ones keep load order)
constexpr int kBalanceBins = 64;        // ... if the geometry has at most this many bins and jobs x bins <= kBalanceWork
constexpr int kBalanceWork = 16384;     // (one thread deals the jobs out)

struct WgradPlanShared {
  int cnt[FLEXMOE_MAX_VEXPERTS], own[FLEXMOE_MAX_VEXPERTS];
  int load[FLEXMOE_MAX_EXPERTS], tiles[FLEXMOE_MAX_EXPERTS], nbuckets[FLEXMOE_MAX_EXPERTS];
  int rank_e[FLEXMOE_MAX_EXPERTS], rank_s[FLEXMOE_MAX_EXPERTS];
  int boff[FLEXMOE_MAX_EXPERTS + 1];
  int4 jobs[kPlanJobsLds];
  int njobs;
  int bal_load[2][kBalanceBins], bal_count[2][kBalanceBins];
};
// One thread: deals the work list (in load order in LDS) out to dst as described above; dst holds -1 everywhere on
// entry.  Returns the positions in use.  A group's list may grow to twice the even share of positions, so that
// 2 seg_rows_max positions always suffice.
__device__ inline int balance_jobs(WgradPlanShared& sh, int which, WgradBalance geo, int seg_tiles, int positions,
                                   int4* __restrict__ dst) {
  const int J = sh.njobs, nb = geo.groups * geo.per_slot;      // position p belongs to bin p % nb
  const int rounds_max = positions / nb;                       // what fits the list
  if (geo.groups <= 1 || nb > kBalanceBins || J * nb > kBalanceWork || rounds_max * nb < J) {
    for (int j = 0; j < J; ++j) dst[j] = sh.jobs[j];
    return J;
  }
  int* load = sh.bal_load[which];
  int* count = sh.bal_count[which];
  for (int c = 0; c < nb; ++c) load[c] = count[c] = 0;
  // jobs per bin at most: twice the even share (once, twice and three times measured the same to 0.5 %)
  const int limit = min(2 * ((J + nb - 1) / nb), rounds_max);
  int rounds = 0;
  for (int j = 0; j < J; ++j) {
    int c = -1;
    for (int q = 0; q < nb; ++q)
      if (count[q] < limit && (c < 0 || load[q] < load[c])) c = q;
    const int4 job = sh.jobs[j];
    const int Te = sh.tiles[job.x];
    const int len = job.z > 1 ? min(seg_tiles, Te - job.y * seg_tiles) : Te;
    load[c] += max(4, (len + 3) & ~3) + 6;               // K tiles of the job + its fixed cost per output tile
    dst[count[c] * nb + c] = job;
    count[c] += 1;
    rounds = max(rounds, count[c]);
  }
  return rounds * nb;
}

// Buckets of the job's expert, copied from the plan into LDS by the workgroup that runs the job.
struct WgradShared {
  int nb;
  int bstart[FLEXMOE_MAX_VEXPERTS], brows[FLEXMOE_MAX_VEXPERTS];
};

// plan: made for product 0 (plan.jobs = dW2's list, plan.jobs_other = dW1's); geo0 / geo1: the two products' geometry.
__device__ __forceinline__ void wgrad_plan_block(const int32_t* __restrict__ voff, const int32_t* __restrict__ owner, int E,
                                                 int V, int seg_tiles, int seg_rows_max, const WgradPlan& plan,
                                                 WgradBalance geo0, WgradBalance geo1) {
  __shared__ WgradPlanShared sh;
  for (int v = threadIdx.x; v < V; v += kGemmThreads) {
    sh.cnt[v] = voff[v + 1] - voff[v];
    sh.own[v] = owner[v];
  }
  for (int e = threadIdx.x; e < E; e += kGemmThreads) {
    sh.load[e] = 0;
    sh.tiles[e] = 0;
    sh.nbuckets[e] = 0;
  }
  __syncthreads();
  for (int v = threadIdx.x; v < V; v += kGemmThreads) {
    atomicAdd(&sh.load[sh.own[v]], sh.cnt[v]);                       // integer sums: order does not matter
    atomicAdd(&sh.tiles[sh.own[v]], (sh.cnt[v] + DK - 1) / DK);
    if (sh.cnt[v] > 0) atomicAdd(&sh.nbuckets[sh.own[v]], 1);
  }
  __syncthreads();
  for (int e = threadIdx.x; e < E; e += kGemmThreads) {
    const int l = sh.load[e];
    int rank = 0;
    for (int o = 0; o < E; ++o) {
      const int lo = sh.load[o];
      rank += (lo > l || (lo == l && o < e)) ? 1 : 0;
    }
    sh.rank_e[rank] = e;
    sh.rank_s[rank] = seg_tiles > 0 ? max(1, (sh.tiles[e] + seg_tiles - 1) / seg_tiles) : 1;
  }
  __syncthreads();
  if (threadIdx.x < kWave) {
    const int lane = threadIdx.x;
    constexpr int kPer = FLEXMOE_MAX_EXPERTS / kWave;
    // prefix over the ranks of the segment counts (and of the segment counts of split experts)
    int sum = 0, sum_split = 0, sum_b = 0;
#pragma unroll
    for (int q = 0; q < kPer; ++q) {
      const int r = lane * kPer + q;
      const int n = r < E ? sh.rank_s[r] : 0;
      sum += n;
      sum_split += n > 1 ? n : 0;
      sum_b += r < E ? sh.nbuckets[r] : 0;                            // by expert id, for the bucket lists
    }
    int incl = sum, incl_split = sum_split, incl_b = sum_b;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
      const int up = __shfl_up(incl, o), up2 = __shfl_up(incl_split, o), up3 = __shfl_up(incl_b, o);
      if (lane >= o) {
        incl += up;
        incl_split += up2;
        incl_b += up3;
      }
    }
    int start = incl - sum, slot = incl_split - sum_split, bo = incl_b - sum_b;
#pragma unroll
    for (int q = 0; q < kPer; ++q) {
      const int r = lane * kPer + q;
      if (r < E) {
        const int n = sh.rank_s[r];
        plan.table[r] = make_int4(sh.rank_e[r], n, slot, 0);
        for (int sg = 0; sg < n; ++sg)
          if (start + sg < seg_rows_max) {
            const int4 job = make_int4(sh.rank_e[r], sg, n, slot);
            if (seg_rows_max <= kPlanJobsLds) {
              sh.jobs[start + sg] = job;
            } else {
              plan.jobs[start + sg] = job;
              plan.jobs_other[start + sg] = job;
            }
          }
        start += n;
        slot += n > 1 ? n : 0;
        sh.boff[r] = bo;
        plan.boff[r] = bo;
        bo += sh.nbuckets[r];
      }
    }
    const int total = __shfl(incl, kWave - 1), total_b = __shfl(incl_b, kWave - 1);
    if (lane == 0) {
      sh.boff[E] = total_b;
      plan.boff[E] = total_b;
      sh.njobs = min(total, seg_rows_max);
      if (seg_rows_max > kPlanJobsLds) plan.njobs[0] = plan.njobs[1] = sh.njobs;
    }
    for (int e = lane; e < E; e += kWave) plan.etiles[e] = sh.tiles[e];
  }
  // the two products' lists, dealt out so that their XCD groups get equal work (one thread of waves 1 and 2 each;
  // the bucket lists below are written meanwhile)
  if (seg_rows_max <= kPlanJobsLds) {
    for (int w = threadIdx.x; w < 2 * seg_rows_max; w += kGemmThreads) {
      plan.jobs[w] = make_int4(-1, 0, 0, 0);
      plan.jobs_other[w] = make_int4(-1, 0, 0, 0);
    }
    __threadfence_block();
    __syncthreads();
    if (threadIdx.x == kWave) plan.njobs[0] = balance_jobs(sh, 0, geo0, seg_tiles, 2 * seg_rows_max, plan.jobs);
    if (threadIdx.x == 2 * kWave) plan.njobs[1] = balance_jobs(sh, 1, geo1, seg_tiles, 2 * seg_rows_max, plan.jobs_other);
  } else {
    __syncthreads();
    for (int w = sh.njobs + threadIdx.x; w < 2 * seg_rows_max; w += kGemmThreads) {
      plan.jobs[w] = make_int4(-1, 0, 0, 0);
      plan.jobs_other[w] = make_int4(-1, 0, 0, 0);
    }
  }
  // bucket lists: a wave per expert, the expert's non-empty buckets in ascending vExpert id
  {
    const int lane = threadIdx.x & (kWave - 1);
    const unsigned long long lt = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    for (int e = threadIdx.x / kWave; e < E; e += kGemmThreads / kWave) {
      int pos0 = sh.boff[e];
      for (int vb = 0; vb < V; vb += kWave) {
        const int v = vb + lane;
        const bool hit = v < V && sh.own[v] == e && sh.cnt[v] > 0;
        const unsigned long long mask = __ballot(hit);
        if (hit) {
          const int pos = pos0 + __popcll(mask & lt);
          plan.bstart[pos] = voff[v];
          plan.brows[pos] = sh.cnt[v];
        }
        pos0 += __popcll(mask);
      }
    }
  }
}

// Everything the kernels of a backward call look up, in one launch: workgroup 0 writes the work list of the
// weight gradients, the others (if any) the row-tile table of the rows products (see rows_plan_block).
__global__ __launch_bounds__(kGemmThreads) void ffn_bwd_plan_kernel(const int32_t* __restrict__ voff,
                                                                    const int32_t* __restrict__ owner, int E, int V,
                                                                    int seg_tiles, int seg_rows_max, WgradPlan plan,
                                                                    WgradBalance geo0, WgradBalance geo1,
                                                                    i32x4* __restrict__ row_tab) {
  if (blockIdx.x == 0) wgrad_plan_block(voff, owner, E, V, seg_tiles, seg_rows_max, plan, geo0, geo1);
  else rows_plan_block(voff, owner, V, row_tab, blockIdx.x - 1, gridDim.x - 1);
}

// The job of work-list position `want` and the buckets of its expert (copied to sh); uniform over the workgroup.
__device__ __forceinline__ WgradJob wgrad_fetch_job(const WgradPlan& plan, int want, WgradShared& sh) {
  const int4 j = plan.jobs[want];
  WgradJob job{j.x, j.y, j.z, j.w};
  job.e = __builtin_amdgcn_readfirstlane(job.e);
  job.seg = __builtin_amdgcn_readfirstlane(job.seg);
  job.nseg = __builtin_amdgcn_readfirstlane(job.nseg);
  job.slot = __builtin_amdgcn_readfirstlane(job.slot);
  if (job.e < 0) return job;
  const int b0 = plan.boff[job.e], nb = plan.boff[job.e + 1] - b0;
  for (int b = threadIdx.x; b < nb; b += blockDim.x) {
    sh.bstart[b] = plan.bstart[b0 + b];
    sh.brows[b] = plan.brows[b0 + b];
  }
  if (threadIdx.x == 0) sh.nb = nb;
  __syncthreads();
  return job;
}

// =============================================================================================
// wgrad_gemm_dma: dW_e[m, n] = sum_{v owned by e, ascending v} sum_{p in bucket v} L[p, m] * R[p, n]
// on the direct-to-LDS pipeline.  Both operands
// are token-major ([tokens, M] and [tokens, NC]), i.e. contraction-strided: their 32-token K tiles
// are copied to LDS as stored and transposed by the LDS reads.  Tokens past the end of a bucket
// (the ragged last K tile of each vExpert, and the padding that rounds the tile count up to the
// pipeline's multiple of 4) are fetched from a row of zeros instead, since direct loads cannot
// be predicated to zero.
// =============================================================================================
__device__ const uint4 kZeroRow[32] = {};

struct DmaSrcTok {
  uint32_t off[kOpLoads];
  int krow[kOpLoads];
  size_t ld;
  __device__ __forceinline__ void init(size_t ld_, int cols_valid) {
    ld = ld_;
    const int w = threadIdx.x >> 6, i = threadIdx.x & 63;
#pragma unroll
    for (int q = 0; q < kOpLoads; ++q) {
      krow[q] = (w * kOpLoads + q) * 2 + (i >> 5);
      const int c = min(dmat_chunk(krow[q], i & 31), cols_valid / 8 - 1);
      off[q] = (uint32_t)(krow[q] * ld + c * 8);
    }
  }
  // `p`: token row 0 of this K tile, first column of the tile; rows >= k_valid come from kZeroRow
  __device__ __forceinline__ void part(lds_byte_t* tile, const bf16_t* __restrict__ p, int k_valid, int q) const {
    const unsigned w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const unsigned lds0 = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)tile) + w * (kOpLoads * 1024);
    const bf16_t* z = (const bf16_t*)kZeroRow + (threadIdx.x & 31) * 8;
    const bf16_t* g = (k_valid >= DK || krow[q] < k_valid) ? p + off[q] : z;
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" FLEXMOE_DMA_CPOL ::"v"(g), "s"(lds0 + q * 1024) : "memory");
  }
};

// Tile sequence of the weight-gradient kernel: 32-token K tiles of the expert's buckets in
// ascending vExpert id, then all-zero tiles up to the padded count.  The position (row pointers of
// both operands, rows left in the bucket) lives in workgroup-uniform values and advances by
// pointer increments; the bucket list in LDS is read only when a bucket is exhausted.
struct WgradIssue {
  const DmaSrcTok& l_src;
  const DmaSrcTok& r_src;
  const bf16_t* L;
  const bf16_t* R;
  const int* bstart;
  const int* brows;
  int M, NC, m0, n0, nb, T;
  int bi, issued;
  const bf16_t* lp;                 // token row 0 of the next K tile, first column of the tile
  const bf16_t* rp;
  int rows_left;                    // rows of bucket bi from that row on
  __device__ __forceinline__ void seek(int bucket, int koff) {
    bi = bucket;
    const int start = __builtin_amdgcn_readfirstlane(bstart[bi]);
    rows_left = __builtin_amdgcn_readfirstlane(brows[bi]) - koff;
    lp = L + ((size_t)start + koff) * M + m0;
    rp = R + ((size_t)start + koff) * NC + n0;
  }
  __device__ __forceinline__ void begin() {}
  __device__ __forceinline__ void part(lds_byte_t* stage, int q) const {
    const int kv = issued < T ? rows_left : 0;
    if (q < kOpLoads) l_src.part(stage, lp, kv, q);
    else r_src.part(stage + kDmaTileBytes, rp, kv, q - kOpLoads);
  }
  __device__ __forceinline__ void end() {
    ++issued;
    if (issued < T) {
      rows_left -= DK;
      lp += (size_t)DK * M;
      rp += (size_t)DK * NC;
      if (rows_left <= 0) seek(min(bi + 1, nb - 1), 0);
    }
  }
};

// Arguments of one weight-gradient GEMM (device pointers; see wgrad_gemm_dma_bf16).
struct WgradDmaArgs {
  const bf16_t* L;
  const bf16_t* R;
  const int32_t* voff;
  const int32_t* owner;
  int E, V, M, NC, m_tiles, n_tiles, seg_tiles, seg_rows_max;
  float* partial;
  WgradPlan plan;
  bf16_t* dw;
};

// One workgroup's tile of a weight-gradient GEMM; `block` is its index in that GEMM's (patched) grid.
__device__ __forceinline__ void wgrad_dma_block(const WgradDmaArgs& p, unsigned block, unsigned char* stage0,
                                                unsigned char* stage1, unsigned char* stage2, unsigned char* stage3,
                                                WgradShared& sh) {
  const bf16_t* __restrict__ L = p.L;
  const bf16_t* __restrict__ R = p.R;
  const int M = p.M, NC = p.NC, m_tiles = p.m_tiles, seg_tiles = p.seg_tiles;
  float* __restrict__ partial = p.partial;
  bf16_t* __restrict__ dw = p.dw;
  // tile grid: rows = (work-list segment, m tile), cols = n tile
  int grow, nt;
  if (!patched_tile(block, p.seg_rows_max * p.m_tiles, p.n_tiles, &grow, &nt)) return;
  const int mt = grow % m_tiles;
  const WgradJob job = wgrad_fetch_job(p.plan, grow / m_tiles, sh);
  if (job.e < 0) return;
  const int nb = sh.nb;

  const int m0 = mt * BM, n0 = nt * BN;
  const int mvalid = min(BM, M - m0), nvalid = min(BN, NC - n0);
  const int wave = threadIdx.x >> 6;
  const int wm = dma_wave_wm(wave), wn = wave & 1, cb0 = dma_wave_cb0(wave);
  DmaAcc acc;
  zero_acc(acc);
  lds_byte_t* s0 = (lds_byte_t*)stage0;

  if (nb > 0) {
    int Te = 0;
    for (int b = 0; b < nb; ++b) Te += (sh.brows[b] + DK - 1) / DK;
    // this job's K tiles [lo, hi) of the expert's sequence, and the bucket / offset where they start
    const int lo = job.nseg > 1 ? job.seg * seg_tiles : 0;
    const int hi = job.nseg > 1 ? min(Te, lo + seg_tiles) : Te;
    int bi = 0, skip = lo;
    while (bi < nb - 1 && skip >= (sh.brows[bi] + DK - 1) / DK) {
      skip -= (sh.brows[bi] + DK - 1) / DK;
      ++bi;
    }
    const int T = hi - lo;
    const int KT = (T + 3) & ~3;                 // padded with all-zero tiles
    DmaSrcTok l_src, r_src;
    l_src.init(M, mvalid);
    r_src.init(NC, nvalid);
    WgradIssue issue{l_src, r_src, L, R, sh.bstart, sh.brows, M, NC, m0, n0, nb, T, 0, 0, nullptr, nullptr, 0};
    issue.seek(bi, skip * DK);
    dma_pipeline<true, true>(s0, (lds_byte_t*)stage1, (lds_byte_t*)stage2, (lds_byte_t*)stage3, acc, issue, KT, wm, cb0);
  }

  float* patch = (float*)stage0 + wave * (16 * 64);
  const int jh = wave >> 2;
  const int col_base = n0 + wn * (NB * 32);
  // whole tiles (every benchmark shape: M and NC are multiples of 256) are stored without predicates
  const bool full = mvalid == BM && nvalid == BN;
  auto valid = [&](const EpiIdx& x) { return (wm + 2 * x.i) * 32 + (x.row_w & 31) < mvalid && col_base + x.col_w < NC; };
  auto none = [](const EpiIdx&) { return make_uint2(0, 0); };
  if (job.nseg == 1) {
    bf16_t* out = dw + (size_t)job.e * M * NC + (size_t)m0 * NC + col_base;      // the wave's block of the tile
    EpiAddr<2> addr;
    addr.init(wm, NC);
    auto to_bf16 = [](const EpiIdx&, float4 c, uint2) { return EpiOut{pack4(c.x, c.y, c.z, c.w), make_uint2(0, 0)}; };
    if (full)
      epilogue_rounds8<false>(patch, jh, acc, none, to_bf16,
                              [&](const EpiIdx& x, const EpiOut& o) { store_nt8(addr.at(out, x), o.a); });   // written once
    else
      epilogue_rounds8<false>(patch, jh, acc, none, to_bf16, [&](const EpiIdx& x, const EpiOut& o) {
        if (valid(x)) store_nt8(addr.at(out, x), o.a);
      });
  } else {
    // one of several segments: the fp32 tile goes to the workspace for wgrad_reduce_kernel
    float* out = partial + (size_t)(job.slot + job.seg) * M * NC + (size_t)m0 * NC + col_base;
    EpiAddr<4> addr;
    addr.init(wm, NC);
    auto as_f32 = [](const EpiIdx&, float4 c, uint2) {
      return EpiOut{make_uint2(__float_as_uint(c.x), __float_as_uint(c.y)), make_uint2(__float_as_uint(c.z), __float_as_uint(c.w))};
    };
    if (full)
      epilogue_rounds8<false>(patch, jh, acc, none, as_f32, [&](const EpiIdx& x, const EpiOut& o) {
        *(uint4*)addr.at(out, x) = make_uint4(o.a.x, o.a.y, o.b.x, o.b.y);
      });
    else
      epilogue_rounds8<false>(patch, jh, acc, none, as_f32, [&](const EpiIdx& x, const EpiOut& o) {
        if (valid(x)) *(uint4*)addr.at(out, x) = make_uint4(o.a.x, o.a.y, o.b.x, o.b.y);
      });
  }
}


__global__ __launch_bounds__(kDmaThreads) void wgrad_gemm_dma_bf16(const WgradDmaArgs p) {
  __shared__ __align__(1024) unsigned char stage0[kDmaStageBytes];
  __shared__ __align__(1024) unsigned char stage1[kDmaStageBytes];
  __shared__ __align__(1024) unsigned char stage2[kDmaStageBytes];
  __shared__ __align__(1024) unsigned char stage3[kDmaStageBytes];
  __shared__ WgradShared sh;
  wgrad_dma_block(p, blockIdx.x, stage0, stage1, stage2, stage3, sh);
}

// =============================================================================================
// wgrad_gemm_persist: the same product on one workgroup per compute unit that walks the output tiles
// (see rows_gemm_persist_bf16 for why): workgroup b takes positions b, b + G, .. of the patched grid
// over (job, m tile) x (n tile), finds each tile's job in the plan with scalar loads, and issues the first
// K tiles of its next output tile while the current K loop drains.  For output matrices that are a whole
// number of 256 x 256 tiles (every benchmark shape; the host falls back to wgrad_gemm_dma_bf16 otherwise),
// so the per-lane load offsets are the same for every tile and only scalars change from tile to tile.
// An expert without tokens contracts four all-zero K tiles (the pipeline's minimum) and stores zeros.
// =============================================================================================
typedef const int __attribute__((address_space(4)))* ConstIntPtr;
typedef int i32x4_t __attribute__((ext_vector_type(4)));
typedef const i32x4_t __attribute__((address_space(4)))* ConstInt4Ptr;

struct WgradIssueV {
  DmaSrcTok l_src, r_src;           // per-lane offsets: the same for every tile of the launch
  ConstIntPtr bstart, brows;        // the expert's bucket list in the plan
  int M, NC, nb, T;
  int bi, issued;
  const bf16_t* lbase;              // L + m0, R + n0: first column of the tile in token row 0
  const bf16_t* rbase;
  const bf16_t* lp;                 // token row 0 of the next K tile, first column of the tile
  const bf16_t* rp;
  int rows_left;                    // rows of bucket bi from that row on
  __device__ __forceinline__ void seek(int bucket, int koff) {
    bi = bucket;
    int start = 0;
    rows_left = 0;
    if (nb > 0) {
      start = bstart[bi];
      rows_left = brows[bi] - koff;
    }
    lp = lbase + ((size_t)start + koff) * M;
    rp = rbase + ((size_t)start + koff) * NC;
  }
  __device__ __forceinline__ void begin() {}
  __device__ __forceinline__ void part(lds_byte_t* stage, int q) const {
    const int kv = issued < T ? rows_left : 0;
    if (q < kOpLoads) l_src.part(stage, lp, kv, q);
    else r_src.part(stage + kDmaTileBytes, rp, kv, q - kOpLoads);
  }
  __device__ __forceinline__ void end() {
    ++issued;
    if (issued < T) {
      rows_left -= DK;
      lp += (size_t)DK * M;
      rp += (size_t)DK * NC;
      if (rows_left <= 0) seek(min(bi + 1, nb - 1), 0);
    }
  }
};

__global__ __launch_bounds__(kDmaThreads) void wgrad_gemm_persist_bf16(const WgradDmaArgs p) {
  __shared__ __align__(1024) unsigned char stage0[kDmaStageBytes];
  __shared__ __align__(1024) unsigned char stage1[kDmaStageBytes];
  __shared__ __align__(1024) unsigned char stage2[kDmaStageBytes];
  __shared__ __align__(1024) unsigned char stage3[kDmaStageBytes];
  lds_byte_t* const s0 = (lds_byte_t*)stage0;
  lds_byte_t* const s1 = (lds_byte_t*)stage1;
  lds_byte_t* const s2 = (lds_byte_t*)stage2;
  lds_byte_t* const s3 = (lds_byte_t*)stage3;
  const ConstInt4Ptr jobs = (ConstInt4Ptr)p.plan.jobs;
  const ConstIntPtr boff = (ConstIntPtr)p.plan.boff, bstart = (ConstIntPtr)p.plan.bstart;
  const ConstIntPtr brows = (ConstIntPtr)p.plan.brows, etiles = (ConstIntPtr)p.plan.etiles;
  const int M = p.M, NC = p.NC, m_tiles = p.m_tiles, n_tiles = p.n_tiles, seg_tiles = p.seg_tiles;
  const int grid_rows = ((ConstIntPtr)p.plan.njobs)[0] * m_tiles;
  const unsigned total = patched_grid(grid_rows, n_tiles);
  const unsigned G = gridDim.x;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = dma_wave_wm(wave), wn = wave & 1, cb0 = dma_wave_cb0(wave);

  struct Tile {
    int e, seg, nseg, slot, m0, n0, KT;
  };
  // the first position from idx on (steps of G) that holds a tile of a job (the list has holes: e = -1)
  auto find = [&](unsigned* idx, int* grow, int* nt) {
    for (; *idx < total; *idx += G)
      if (patched_tile(*idx, grid_rows, n_tiles, grow, nt) && jobs[*grow / m_tiles][0] >= 0) return true;
    return false;
  };
  // tile -> its description and its K-tile sequence (scalars only)
  auto describe = [&](int grow, int nt, Tile* t, WgradIssueV* is) {
    const i32x4_t job = jobs[grow / m_tiles];
    t->e = job[0];
    t->seg = job[1];
    t->nseg = job[2];
    t->slot = job[3];
    t->m0 = (grow % m_tiles) * BM;
    t->n0 = nt * BN;
    const int b0 = boff[t->e], nb = boff[t->e + 1] - b0, Te = etiles[t->e];
    // this job's K tiles [lo, hi) of the expert's sequence, and the bucket / offset where they start
    const int lo = t->nseg > 1 ? t->seg * seg_tiles : 0;
    const int hi = t->nseg > 1 ? min(Te, lo + seg_tiles) : Te;
    int bi = 0, skip = lo;
    while (bi < nb - 1 && skip >= (brows[b0 + bi] + DK - 1) / DK) {
      skip -= (brows[b0 + bi] + DK - 1) / DK;
      ++bi;
    }
    const int T = hi - lo;
    t->KT = max(4, (T + 3) & ~3);               // padded with all-zero tiles
    is->bstart = bstart + b0;
    is->brows = brows + b0;
    is->nb = nb;
    is->T = T;
    is->issued = 0;
    is->lbase = p.L + t->m0;
    is->rbase = p.R + t->n0;
    is->seek(bi, skip * DK);
  };

  unsigned idx = blockIdx.x;
  int grow, nt;
  if (!find(&idx, &grow, &nt)) return;
  WgradIssueV issue;
  issue.l_src.init(M, BM);
  issue.r_src.init(NC, BN);
  issue.M = M;
  issue.NC = NC;
  Tile t;
  describe(grow, nt, &t, &issue);
  dma_prefetch3(s0, s1, s2, issue);
  float* const patch = (float*)stage3 + wave * (16 * 64);      // wave-private, 4 KB; stage 3 is the one the next tile has not touched yet

  TilePhases phases;
  for (;;) {
    phases.start();
    DmaAcc acc;
    zero_acc(acc);
    unsigned nidx = idx + G;
    int ngrow, nnt;
    const bool has_next = find(&nidx, &ngrow, &nnt);
    // (none: this tile's first K tiles once more, waited for below and never used)
    WgradIssueV next = issue;
    Tile tn;
    describe(has_next ? ngrow : grow, has_next ? nnt : nt, &tn, &next);
    dma_pipeline_cont<true, true>(s0, s1, s2, s3, acc, issue, t.KT, next, wm, cb0, [&]() { phases.first_barrier(); },
                                  [](WgradIssueV&) {});
    phases.k_done();

    const int col_base = t.n0 + wn * (NB * 32);
    auto none = [](const EpiIdx&) { return make_uint2(0, 0); };
    if (t.nseg == 1) {
      bf16_t* out = p.dw + (size_t)t.e * M * NC + (size_t)t.m0 * NC + col_base;      // the wave's block of the tile
      EpiAddr<2> addr;
      addr.init(wm, NC);
      epilogue_rounds8<false>(
          patch, wave >> 2, acc, none,
          [](const EpiIdx&, float4 c, uint2) { return EpiOut{pack4(c.x, c.y, c.z, c.w), make_uint2(0, 0)}; },
          [&](const EpiIdx& x, const EpiOut& o) { store_nt8(addr.at(out, x), o.a); });      // written once
    } else {
      // one of several segments: the fp32 tile goes to the workspace for wgrad_reduce_kernel
      float* out = p.partial + (size_t)(t.slot + t.seg) * M * NC + (size_t)t.m0 * NC + col_base;
      EpiAddr<4> addr;
      addr.init(wm, NC);
      epilogue_rounds8<false>(
          patch, wave >> 2, acc, none,
          [](const EpiIdx&, float4 c, uint2) {
            return EpiOut{make_uint2(__float_as_uint(c.x), __float_as_uint(c.y)),
                          make_uint2(__float_as_uint(c.z), __float_as_uint(c.w))};
          },
          [&](const EpiIdx& x, const EpiOut& o) { *(uint4*)addr.at(out, x) = make_uint4(o.a.x, o.a.y, o.b.x, o.b.y); });
    }
    phases.tile_done(4, !has_next);
    if (!has_next) break;
    t = tn;
    issue = next;
    idx = nidx;
    grow = ngrow;
    nt = nnt;
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);                  // vmcnt(0): nothing may still be landing in LDS when the workgroup ends
}

// dW_e = sum of the expert's partial tiles in segment order, for the experts that were split.
// Grid: (element blocks of the [M, NC] matrix, load rank); `table` as left by the GEMM kernel.
__global__ __launch_bounds__(kGemmThreads) void wgrad_reduce_kernel(const int4* __restrict__ table, int M, int NC,
                                                                    const float* __restrict__ partial,
                                                                    bf16_t* __restrict__ dw) {
  const int4 t = table[blockIdx.y];             // {expert, segments, first slot}
  if (t.y <= 1) return;
  const size_t n4 = (size_t)M * NC / 4;
  const float4* p = (const float4*)(partial + (size_t)t.z * M * NC);
  uint2* out = (uint2*)(dw + (size_t)t.x * M * NC);
  for (size_t i = (size_t)blockIdx.x * kGemmThreads + threadIdx.x; i < n4; i += (size_t)gridDim.x * kGemmThreads) {
    float4 s4 = p[i];
    for (int sgm = 1; sgm < t.y; ++sgm) {
      const float4 v = p[(size_t)sgm * n4 + i];
      s4.x += v.x; s4.y += v.y; s4.z += v.z; s4.w += v.w;
    }
    store_nt8((bf16_t*)(out + i), pack4(s4.x, s4.y, s4.z, s4.w));   // written once, like the unsplit experts' tiles
  }
}

}  // namespace flexmoe
