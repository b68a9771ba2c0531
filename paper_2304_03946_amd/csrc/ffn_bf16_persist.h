// Persistent rows kernels: one workgroup per compute unit walks its share of the output tiles, and the
// operand loads of a tile's successor are issued while the tile's own K loop drains.
// Part of the bf16 expert-FFN kernels; included by ffn_bf16.hip only (one translation unit).
#pragma once
#include "common.h"
#include "ffn_bf16_tile.h"
#include "ffn_bf16_dma.h"
namespace flexmoe {
// =============================================================================================
// Why: with 128 KB of LDS stages and 256 accumulator registers per lane a compute unit holds one
// workgroup, so whatever a workgroup does before its first MFMA and after its last one is time the matrix
// pipe idles: workgroup start-up, finding the tile in the bucket list, the first operand tiles' trip
// from memory.  Here a launch has (at most) 256 workgroups; workgroup b takes the grid positions
// b, b + 256, b + 512, .. of the XCD-aware patch order (patched_tile: position % 8 is the XCD, so every
// round of 256 positions is eight neighbouring patches, one per XCD, exactly the schedule the hardware
// dispatcher produces for a one-tile-per-workgroup grid, but in lockstep).  Row tiles are found in a
// table that rows_plan_kernel writes once per call ({first row, rows, expert} per 256-row tile of the
// bucket list), read with scalar loads through the constant address space.
//
// The last, partly filled round of a product with a long contraction is cut along K as in the
// one-tile-per-workgroup kernels (lookup_row_tile): here the tail tiles are left out of the walk over
// the grid and their S x tail_tiles K segments form one more round, workgroup b taking segment
// (b % S) of tail tile b / S.
// =============================================================================================
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef const i32x4 __attribute__((address_space(4)))* RowTabPtr;

// tab[0] = {row tiles of the bucket list, 0, 0, 0}; tab[1 + t] = {first row, rows, expert, 0} of row tile t.
__host__ __device__ inline size_t rows_tab_bytes(int row_tiles_max) { return ((size_t)row_tiles_max + 1) * sizeof(i32x4); }

// Workgroup `block` of `nblocks` that fill the table (each derives the bucket prefix again and writes its share of the rows).
__device__ __forceinline__ void rows_plan_block(const int32_t* __restrict__ voff, const int32_t* __restrict__ owner, int V,
                                                i32x4* __restrict__ tab, int block, int nblocks) {
  __shared__ int cum[FLEXMOE_MAX_VEXPERTS + 1];      // cum[v] = row tiles before bucket v
  __shared__ int wsum[kGemmThreads / kWave];
  // two buckets per thread, inclusive scan over the workgroup
  const int t = threadIdx.x, lane = t & (kWave - 1), wave = t / kWave;
  int c0 = 0, c1 = 0;
  if (2 * t < V) c0 = (voff[2 * t + 1] - voff[2 * t] + BM - 1) / BM;
  if (2 * t + 1 < V) c1 = (voff[2 * t + 2] - voff[2 * t + 1] + BM - 1) / BM;
  int incl = c0 + c1;
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    const int up = __shfl_up(incl, o);
    if (lane >= o) incl += up;
  }
  if (lane == kWave - 1) wsum[wave] = incl;
  __syncthreads();
  int before = 0;
  for (int w = 0; w < wave; ++w) before += wsum[w];
  const int excl = before + incl - c0 - c1;
  if (t == 0) cum[0] = 0;
  if (2 * t + 1 <= V) cum[2 * t + 1] = excl + c0;
  if (2 * t + 2 <= V) cum[2 * t + 2] = excl + c0 + c1;
  __syncthreads();
  const int rows_act = cum[V];
  if (block == 0 && t == 0) tab[0] = i32x4{rows_act, 0, 0, 0};
  for (int rt = block * kGemmThreads + t; rt < rows_act; rt += nblocks * kGemmThreads) {
    int lo = 0, hi = V;                              // last v with cum[v] <= rt (empty buckets share a value: take the last)
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (cum[mid] <= rt) lo = mid;
      else hi = mid;
    }
    const int row0 = voff[lo] + (rt - cum[lo]) * BM;
    tab[1 + rt] = i32x4{row0, min(BM, voff[lo + 1] - row0), owner[lo], 0};
  }
}

__global__ __launch_bounds__(kGemmThreads) void rows_plan_kernel(const int32_t* __restrict__ voff,
                                                                 const int32_t* __restrict__ owner, int V,
                                                                 i32x4* __restrict__ tab) {
  rows_plan_block(voff, owner, V, tab, blockIdx.x, gridDim.x);
}

// The walk of one product's tiles (all values uniform over the launch).
struct TileSeq {
  int rows_act, col_tiles;
  int S, r_split, tail_tiles;      // split of the last round: S == 1: none
  unsigned n_main, total;
};
struct TileId {
  int rt, ct, seg, nseg, slot;
};
__device__ __forceinline__ TileSeq make_tile_seq(int rows_act, int col_tiles, bool may_split, int k_tiles) {
  TileSeq q;
  q.rows_act = rows_act;
  q.col_tiles = col_tiles;
  q.n_main = patched_grid(rows_act, col_tiles);
  q.S = 1;
  q.r_split = rows_act;
  q.tail_tiles = 0;
  if (may_split) {
    const int full = rows_act * col_tiles / kSplitUnits;
    const int r_split = full * kSplitUnits / col_tiles;
    const int tail_tiles = (rows_act - r_split) * col_tiles;
    const int S = split_factor(full, tail_tiles, k_tiles);
    if (S > 1) {
      q.S = S;
      q.r_split = r_split;
      q.tail_tiles = tail_tiles;
    }
  }
  q.total = q.n_main + (q.S > 1 ? (unsigned)kSplitUnits : 0u);
  return q;
}
__device__ __forceinline__ bool decode_tile(const TileSeq& q, unsigned idx, TileId* id) {
  if (idx < q.n_main) {
    if (!patched_tile(idx, q.rows_act, q.col_tiles, &id->rt, &id->ct)) return false;
    if (id->rt >= q.r_split) return false;           // tail tile: contracted in segments, below
    id->seg = 0;
    id->nseg = 1;
    id->slot = 0;
    return true;
  }
  const int y = (int)(idx - q.n_main);
  if (y >= q.tail_tiles * q.S) return false;
  const int tt = y / q.S;
  id->rt = q.r_split + tt / q.col_tiles;
  id->ct = tt % q.col_tiles;
  id->seg = y % q.S;
  id->nseg = q.S;
  id->slot = tt * q.S + id->seg;
  return true;
}
// The first position from idx on (in steps of G) that holds a tile; false: none left.
__device__ __forceinline__ bool find_tile(const TileSeq& q, unsigned* idx, unsigned G, TileId* id) {
  for (; *idx < q.total; *idx += G)
    if (decode_tile(q, *idx, id)) return true;
  return false;
}

// Profiling build only (-DFLEXMOE_TILE_PHASES, paper_2304_03946_amd/tile_phases.py): per workgroup, the 100 MHz
// clock ticks spent from a tile's start to its first barrier ("top": the previous epilogue's stragglers, the wait
// for the first K tile), in the K loop and in the epilogue, and the tiles done; one set per kind of rows product.
#ifdef FLEXMOE_TILE_PHASES
__device__ unsigned long long g_tile_phases[5][256][4];      // [GEMM1, GEMM2, dH, dXp, weight gradient][workgroup][top, K loop, epilogue, tiles]
struct TilePhases {
  unsigned long long top = 0, kloop = 0, epi = 0, n = 0, c0 = 0, c1 = 0, c2 = 0;
  __device__ __forceinline__ void start() { c0 = c1 = wall_clock64(); }
  __device__ __forceinline__ void first_barrier() { c1 = wall_clock64(); }
  __device__ __forceinline__ void k_done() { c2 = wall_clock64(); }
  __device__ __forceinline__ void tile_done(int kind, bool last) {
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    const unsigned long long c3 = wall_clock64();
    top += c1 - c0; kloop += c2 - c1; epi += c3 - c2; n += 1;
    if (last && threadIdx.x == 0) {
      g_tile_phases[kind][blockIdx.x][0] = top; g_tile_phases[kind][blockIdx.x][1] = kloop;
      g_tile_phases[kind][blockIdx.x][2] = epi; g_tile_phases[kind][blockIdx.x][3] = n;
    }
  }
};
#else
struct TilePhases {
  __device__ __forceinline__ void start() {}
  __device__ __forceinline__ void first_barrier() {}
  __device__ __forceinline__ void k_done() {}
  __device__ __forceinline__ void tile_done(int, bool) {}
};
#endif
template <typename WSrc> struct RowsIssueV {
  DmaSrc a_src;
  WSrc w_src;
  int k_next;
  __device__ __forceinline__ void begin() {}
  __device__ __forceinline__ void part(lds_byte_t* stage, int q) const {
    if (q < kOpLoads) a_src.part(stage, k_next, q);
    else w_src.part(stage + kDmaTileBytes, k_next, q - kOpLoads);
  }
  __device__ __forceinline__ void end() { k_next += DK; }
};

template <bool WT> struct RowsWSrc {
  typedef DmaSrcT type;
};
template <> struct RowsWSrc<true> {
  typedef DmaSrc type;
};

// Arguments: RowsDmaArgs (split_partial: null = no splitting; normal_grid unused) plus the row-tile table.
// GATHER: p.gsrc holds the rows of `in` to read (rows gathered on load).
template <bool WT, int EPI, int ACT, bool GATHER>
__global__ __launch_bounds__(kDmaThreads) void rows_gemm_persist_bf16(const RowsDmaArgs p, const i32x4* row_tab) {
  __shared__ __align__(1024) unsigned char stage0[kDmaStageBytes];
  __shared__ __align__(1024) unsigned char stage1[kDmaStageBytes];
  __shared__ __align__(1024) unsigned char stage2[kDmaStageBytes];
  __shared__ __align__(1024) unsigned char stage3[kDmaStageBytes];
  constexpr bool kLut = epilogue_uses_lut<EPI, ACT>();
  __shared__ __align__(1024) unsigned char lut_lds[kLut ? kLutBytes : 16];
  __shared__ int smap_lds[EPI == EPI_PLAIN ? BM : 1];
  lds_byte_t* const s0 = (lds_byte_t*)stage0;
  lds_byte_t* const s1 = (lds_byte_t*)stage1;
  lds_byte_t* const s2 = (lds_byte_t*)stage2;
  lds_byte_t* const s3 = (lds_byte_t*)stage3;
  typedef typename RowsWSrc<WT>::type WSrc;
  typedef RowsIssueV<WSrc> Issue;

  const RowTabPtr tab = (RowTabPtr)row_tab;
  const int K = p.K, NC = p.NC;
  const TileSeq seq = make_tile_seq(tab[0][0], p.col_tiles, EPI == EPI_PLAIN && p.split_partial != nullptr, K / DK);
  const unsigned G = gridDim.x;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = dma_wave_wm(wave), wn = wave & 1, cb0 = dma_wave_cb0(wave);

  // tile -> operand sources and the K range [k0, k0 + 32 KT)
  auto fetch_tile = [&](const TileId& id) {
    const i32x4 d = tab[1 + id.rt];
    RowTile t;
    t.row0 = d[0];
    t.rows_valid = d[1];
    t.e = d[2];
    t.n0 = id.ct * BN;
    t.cols_valid = min(BN, NC - t.n0);
    t.seg = id.seg;
    t.nseg = id.nseg;
    t.slot = id.slot;
    return t;
  };
  auto make_issue = [&](const RowTile& t) {
    Issue is;
    if constexpr (GATHER) is.a_src.init_gather(p.in, K, p.gsrc + t.row0, p.gk, t.rows_valid);
    else is.a_src.init(p.in + (size_t)t.row0 * K, K, t.rows_valid);
    const bf16_t* w_e = p.w + (size_t)t.e * K * NC;
    if constexpr (WT) is.w_src.init(w_e + (size_t)t.n0 * K, K, t.cols_valid);
    else is.w_src.init(w_e + t.n0, NC, t.cols_valid);
    is.k_next = t.nseg > 1 ? t.seg * (K / DK / t.nseg) * DK : 0;
    return is;
  };

  unsigned idx = blockIdx.x;
  TileId id;
  if (!find_tile(seq, &idx, G, &id)) return;
  const lds_byte_t* lut = nullptr;
  if (kLut) lut = (const lds_byte_t*)lut_lds;
  if (kLut && wave < 4) {
    // the table rides in front of the first operand tiles (four waves fetch a quarter each): its direct loads are the
    // oldest in those waves' queues, so the first wait of the K loop covers them and its barrier publishes them
    const unsigned lds0 = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)lut) + wave * (kLutBytes / 4);
    const unsigned char* g = (const unsigned char*)g_act_lut[ACT == FLEXMOE_GELU_ERF ? 0 : 1] + wave * (kLutBytes / 4) +
                             (threadIdx.x & 63) * 16;
#pragma unroll
    for (int q = 0; q < kLutBytes / 4 / 1024; ++q) {
      const unsigned char* gq = g + q * 1024;
      asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" FLEXMOE_DMA_CPOL ::"v"(gq), "s"(lds0 + q * 1024) : "memory");
    }
  }
  RowTile t = fetch_tile(id);
  Issue issue = make_issue(t);
  dma_prefetch3(s0, s1, s2, issue);
  float* const patch = (float*)stage3 + wave * (16 * 64);      // wave-private, 4 KB; stage 3 is the one the next tile has not touched yet

  TilePhases phases;
  for (;;) {
    phases.start();
    DmaAcc acc;
    zero_acc(acc);
    // the workgroup's next tile
    unsigned nidx = idx + G;
    TileId nid;
    const bool has_next = find_tile(seq, &nidx, G, &nid);
    // (none: the loads of this tile's first K tiles once more, waited for below and never used)
    const RowTile tn = has_next ? fetch_tile(nid) : t;
    Issue next;
    if constexpr (GATHER) next = make_issue(tn);       // its index loads share the operand tiles' queue: up here, where little is in flight
    const int KT = K / DK / t.nseg;
    dma_pipeline_cont<false, !WT>(
        s0, s1, s2, s3, acc, issue, KT, next, wm, cb0,
        [&]() {
          phases.first_barrier();
          if (EPI == EPI_PLAIN && p.scatter_rows && t.nseg == 1 && threadIdx.x < BM)
            smap_lds[threadIdx.x] = p.scatter_rows[t.row0 + min((int)threadIdx.x, t.rows_valid - 1)];
        },
        [&](Issue& nx) {
          if constexpr (!GATHER) nx = make_issue(tn);
        });
    phases.k_done();
    if (EPI == EPI_PLAIN && t.nseg > 1) {
      // one K segment of a split tile: fp32 partial tile (all 256 x 256 entries) for the reduce kernel
      float* out = p.split_partial + (size_t)t.slot * (BM * BN);
      epilogue_rounds8<false>(
          patch, wave >> 2, acc, [](const EpiIdx&) { return make_uint2(0, 0); },
          [](const EpiIdx&, float4 c, uint2) {
            return EpiOut{make_uint2(__float_as_uint(c.x), __float_as_uint(c.y)),
                          make_uint2(__float_as_uint(c.z), __float_as_uint(c.w))};
          },
          [&](const EpiIdx& x, const EpiOut& o) {
            const int lrow = (wm + 2 * x.i) * 32 + (x.row_w & 31);
            *(uint4*)(out + lrow * BN + wn * (NB * 32) + x.col_w) = make_uint4(o.a.x, o.a.y, o.b.x, o.b.y);
          });
    } else {
      const lds_int_t* smap = (EPI == EPI_PLAIN && p.scatter_rows) ? (const lds_int_t*)smap_lds : nullptr;
      rows_epilogue<EPI, ACT, kLut, 8>((float*)stage3, (float*)stage3, acc, p.bias, NC, t.row0, t.rows_valid, t.e, t.n0,
                                    p.hpre_in, p.out0, p.out1, lut, smap);
    }
    phases.tile_done((WT ? 2 : 0) + (EPI == EPI_PLAIN ? 1 : 0), !has_next);
    if (!has_next) break;
    t = tn;
    issue = next;
    idx = nidx;
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);                  // vmcnt(0): nothing may still be landing in LDS when the workgroup ends
}

}  // namespace flexmoe
