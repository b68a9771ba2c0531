// Direct-to-LDS pipeline (global_load_lds): operand sources, the K loop in its one-tile and its continuing form, the sum of the split last round.
// Part of the bf16 expert-FFN kernels; included by ffn_bf16.hip only (one translation unit).
#pragma once
#include "common.h"
#include "ffn_bf16_tile.h"
namespace flexmoe {
// =============================================================================================
// rows_gemm_dma: the same product for operands that are both contraction-contiguous
// (In [rows, K], W_e [NC, K]) and K a multiple of 128, with global -> LDS direct loads
// (global_load_lds, 16 bytes per lane, no register staging, no LDS store instructions).
// Four LDS stages of a 32-wide K tile (2 x 16 KB each): while tile t is multiplied, tiles
// t+1..t+3 are landed or in flight and tile t+4 is issued half-way through the step.  A direct load writes lane i's 16 bytes at
// the wave's LDS base + 16*i, so one instruction fills 16 rows x 64 bytes; the bank swizzle
// (16-byte chunk index XOR (row>>2)&3) is applied by choosing which global chunk a lane fetches.
// =============================================================================================
// The tile is worked on by eight waves, two per SIMD: wave w owns rows (wm + 2 i) * 32, i < 4, and the two
// 32-column blocks cb0, cb0 + 1 with wm = (w >> 1) & 1, cb0 = (w & 1) * 4 + (w >> 2) * 2 -- 128 x 64 outputs, 128
// accumulator registers.  With one wave per SIMD (128 x 128 outputs each) nothing can issue while that wave
// waits for LDS data, a barrier or its loads; with two, the other wave's MFMAs fill the gap (measured on the
// stripped K loop with random operands and everything in L2: 1.34 -> 1.48 PFLOP/s).
constexpr int DK = 32;
constexpr int kDmaStages = 4;
constexpr int kDmaWaves = 8;
constexpr int kDmaThreads = kDmaWaves * kWave;
constexpr int NBW = 2;                                 // 32-column blocks per wave
constexpr int kOpLoads = 16 / kDmaWaves;               // direct loads (1 KB) per wave and 16 KB operand tile
__device__ __forceinline__ int dma_wave_wm(int w) { return (w >> 1) & 1; }
__device__ __forceinline__ int dma_wave_cb0(int w) { return (w & 1) * 4 + (w >> 2) * 2; }
constexpr int kDmaTileBytes = 256 * DK * 2;            // one operand tile: 16 KB
constexpr int kDmaStageBytes = 2 * kDmaTileBytes;      // A + B

__device__ __forceinline__ int dma_off(int row, int c) { return row * (DK * 2) + ((c ^ ((row >> 2) & 3)) << 4); }

struct DmaSrc {
  const bf16_t* base;
  uint32_t off[kOpLoads];
  __device__ __forceinline__ void init(const bf16_t* b, size_t ld, int rows_valid) {
    base = b;
    const int tid = opaque_tid();
    const int w = tid >> 6, i = tid & 63;
#pragma unroll
    for (int q = 0; q < kOpLoads; ++q) {
      const int row = (w * kOpLoads + q) * 16 + (i >> 2);
      const int c = (i & 3) ^ ((row >> 2) & 3);
      off[q] = (uint32_t)(min(row, rows_valid - 1) * ld + c * 8);
    }
  }
  // The same tile with its rows gathered: tile row r is row rows[r] / k of the matrix at b (the
  // expert-wise layout transformation done on the fly: rows = the bucket's slice of `src`).
  __device__ __forceinline__ void init_gather(const bf16_t* b, size_t ld, const int32_t* __restrict__ rows, int k,
                                              int rows_valid) {
    base = b;
    const int tid = opaque_tid();
    const int w = tid >> 6, i = tid & 63;
#pragma unroll
    for (int q = 0; q < kOpLoads; ++q) {
      const int row = (w * kOpLoads + q) * 16 + (i >> 2);
      const int c = (i & 3) ^ ((row >> 2) & 3);
      off[q] = (uint32_t)((size_t)(rows[min(row, rows_valid - 1)] / k) * ld + c * 8);
    }
  }
  // Fills the 16 KB LDS tile at `tile` with K columns k0..k0+31 of the operand's 256 rows.
  // The direct load is issued from inline assembly (M0 = LDS byte address of the wave's 1 KB
  // slice, lane i lands at M0 + 16*i): the compiler's wait-count insertion cannot tell which LDS
  // stage a direct load writes and would wait for every outstanding load before any LDS read;
  // here the waits are placed by hand (wait_vmcnt_le) before the barrier that publishes a stage.
  // q-th of the wave's kOpLoads direct loads of one tile
  __device__ __forceinline__ void part(lds_byte_t* tile, int k0, int q) const {
    const unsigned w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const unsigned lds0 = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)tile) + w * (kOpLoads * 1024);
    const bf16_t* g = base + k0 + off[q];
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" FLEXMOE_DMA_CPOL ::"v"(g), "s"(lds0 + q * 1024) : "memory");
  }
};

// Operand stored [K, ld] with the output index contiguous (the forward weights W_e [K, NC]): the
// 32 x 256 tile is copied to LDS as it lies in memory, one k-row = 512 bytes = 32 chunks, two
// k-rows per direct-load instruction, and transposed on the way out of LDS by ds_read_tr16_b64.
// Chunk index XOR (k & 3) << 2 keeps those transposing reads free of bank conflicts.  Columns
// past cols_valid are clamped to the last valid 8-column chunk.
typedef short s16x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ int dmat_chunk(int krow, int c) { return c ^ ((krow & 3) << 2); }

struct DmaSrcT {
  const bf16_t* base;     // first contraction row, first column of the tile
  uint32_t off[kOpLoads];
  size_t ld;
  __device__ __forceinline__ void init(const bf16_t* b, size_t ld_, int cols_valid) {
    base = b;
    ld = ld_;
    const int tid = opaque_tid();
    const int w = tid >> 6, i = tid & 63;
#pragma unroll
    for (int q = 0; q < kOpLoads; ++q) {
      const int krow = (w * kOpLoads + q) * 2 + (i >> 5);
      const int c = min(dmat_chunk(krow, i & 31), cols_valid / 8 - 1);
      off[q] = (uint32_t)(krow * ld + c * 8);
    }
  }
  __device__ __forceinline__ void part(lds_byte_t* tile, int k0, int q) const {
    const unsigned w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const unsigned lds0 = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)tile) + w * (kOpLoads * 1024);
    const bf16_t* g = base + (size_t)k0 * ld + off[q];
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" FLEXMOE_DMA_CPOL ::"v"(g), "s"(lds0 + q * 1024) : "memory");
  }
};

// MFMA fragment (8 consecutive k of output column nb0 + lane%32, k = 16*ks + 8*(lane/32) ..) from
// a [32 k][256 n] tile.  ds_read_tr16_b64 works on groups of 16 lanes: lanes 4m..4m+3 of a group
// address 16 consecutive elements of row m (4 each) and lane i of the group receives column i of
// those four rows.  So lane L (group g = L/16, i = L%16) points at row k' + i/4, columns
// nb0 + 16*(g%2) + 4*(i%4), with k' = 16*ks + 8*(g/2) (+4 for the second read).
__device__ __forceinline__ bf16x8 dmat_read_frag(const lds_byte_t* tile, int nb0, int ks) {
  const int L = threadIdx.x & 63;
  const int g = L >> 4, i = L & 15;
  const int col = nb0 + 16 * (g & 1) + 4 * (i & 3);
  const int k_lo = 16 * ks + 8 * (g >> 1) + (i >> 2);
  const int k_hi = k_lo + 4;
  const int a_lo = k_lo * 512 + (dmat_chunk(k_lo, col >> 3) << 4) + ((col & 7) << 1);
  const int a_hi = k_hi * 512 + (dmat_chunk(k_hi, col >> 3) << 4) + ((col & 7) << 1);
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(tile + a_lo));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(tile + a_hi));
  typedef short s16x8 __attribute__((ext_vector_type(8)));
  const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, v);
}

// s_waitcnt vmcnt(n) only (expcnt / lgkmcnt fields left at "no wait").
template <int N> __device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit field");
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}
// Returns once at most `tiles` of the most recently issued K tiles (2 kOpLoads direct loads per wave each) are in flight.
template <int TILES> __device__ __forceinline__ void wait_tiles_in_flight() { wait_vmcnt<2 * kOpLoads * TILES>(); }

struct DmaFrags {
  Frag8 a[MB], b[NBW];
};
typedef f32x16 DmaAcc[MB][NBW];
__device__ __forceinline__ void zero_acc(DmaAcc& acc) {
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NBW; ++j)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.f;
}
// TRA / TRB: the operand's LDS tile is [k][256] (transposing reads) instead of [256][k].
template <bool TRA, bool TRB>
__device__ __forceinline__ void dma_read_frags(DmaFrags& f, const lds_byte_t* stage, int ks, int wm, int cb0) {
  const int lane = threadIdx.x & 63;
  const int r = lane & 31, h = lane >> 5;
  const lds_byte_t* As = stage;
  const lds_byte_t* Bs = stage + kDmaTileBytes;
#pragma unroll
  for (int i = 0; i < MB; ++i) {
    if (TRA) f.a[i].v = dmat_read_frag(As, (wm + 2 * i) * 32, ks);
    else f.a[i].v = *(const __attribute__((address_space(3))) bf16x8*)(As + dma_off((wm + 2 * i) * 32 + r, 2 * ks + h));
  }
#pragma unroll
  for (int j = 0; j < NBW; ++j) {
    if (TRB) f.b[j].v = dmat_read_frag(Bs, (cb0 + j) * 32, ks);
    else f.b[j].v = *(const __attribute__((address_space(3))) bf16x8*)(Bs + dma_off((cb0 + j) * 32 + r, 2 * ks + h));
  }
}

// One K tile (two 16-wide k steps).  On entry f0 holds the fragments of (tile kt, k step 0).
// The barrier sits between the two k steps: before it the wave has fetched everything it needs
// from `cur`, so after it `cur` is free for tile kt+4; and tile kt+1 is published, so its first
// fragments can be fetched while the second k step's MFMAs run -- no LDS latency after the barrier.
// The direct loads are spread evenly between the MFMAs, one after every four (128 cycles of
// matrix-pipe work): the waves share one address path, and a wave that issues its loads back
// to back leaves its matrix pipe idle while it queues there.  So a tile's 2 kOpLoads loads per wave go
// out in two halves: the first operand's (of tile kt+4) after the barrier of step kt (into `cur`, just
// freed), the second operand's before the barrier of step kt+1 (into that step's `prev`).
// Issue: begin() prepares the next tile in sequence, part(stage, q) starts its q-th direct load
// (q = 0 .. 2 kOpLoads - 1) into `stage`, end() moves on to the tile after it.
// PRE: tile kt+3 exists (its second half is issued here).  POST: tile kt+4 exists.
// NEXT: tile kt+1 exists; WAIT = how many younger tiles may still be in flight once this wave's
// part of tile kt+1 has landed.
// `issue` serves the first half of the step (PRE), `issue_post` the second (POST): the same object inside a
// tile sequence, two different ones where the sequence of the workgroup's next output tile takes over.
template <bool TRA, bool TRB, bool PRE, bool POST, int WAIT, bool NEXT, typename Issue, typename IssuePost>
__device__ __forceinline__ void dma_step(lds_byte_t* prev, lds_byte_t* cur, const lds_byte_t* nxt, DmaAcc& acc,
                                         DmaFrags& f0, DmaFrags& f1, Issue& issue, IssuePost& issue_post, int wm,
                                         int cb0) {
  constexpr int kEvery = MB / kOpLoads;      // a load after every kEvery-th group of NBW MFMAs
  dma_read_frags<TRA, TRB>(f1, cur, 1, wm, cb0);
#pragma unroll
  for (int i = 0; i < MB; ++i) {
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int j = 0; j < NBW; ++j)
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f0.b[j].v, f0.a[i].v, acc[i][j], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    if (PRE && i % kEvery == kEvery - 1) issue.part(prev, kOpLoads + i / kEvery);
  }
  if (PRE) issue.end();
  __builtin_amdgcn_sched_barrier(0);     // everything above is queued before the wave goes to wait
  if (NEXT) wait_tiles_in_flight<WAIT>();
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
  if (NEXT) dma_read_frags<TRA, TRB>(f0, nxt, 0, wm, cb0);
  if (POST) issue_post.begin();
#pragma unroll
  for (int i = 0; i < MB; ++i) {
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int j = 0; j < NBW; ++j)
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f1.b[j].v, f1.a[i].v, acc[i][j], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    if (POST && i % kEvery == kEvery - 1) issue_post.part(cur, i / kEvery);
  }
}

// The whole K loop: KT tiles (a multiple of 4) through the four stages; the last four tiles,
// which have nothing left to prefetch, run as a peeled tail so that the steady-state loop body is
// branch-free.
template <bool TRA, bool TRB, typename Issue>
__device__ __forceinline__ void dma_pipeline(lds_byte_t* s0, lds_byte_t* s1, lds_byte_t* s2, lds_byte_t* s3,
                                             DmaAcc& acc, Issue& issue, int KT, int wm, int cb0) {
  lds_byte_t* const stages[4] = {s0, s1, s2, s3};
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    issue.begin();
#pragma unroll
    for (int q = 0; q < (t < 3 ? 2 * kOpLoads : kOpLoads); ++q) issue.part(stages[t], q);   // tile 3: first half only
    if (t < 3) issue.end();
  }
  wait_vmcnt<5 * kOpLoads>();                          // tile 0 has landed (two and a half tiles younger)
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
  DmaFrags f0, f1;
  dma_read_frags<TRA, TRB>(f0, s0, 0, wm, cb0);
  for (int kt = 0; kt < KT - 4; kt += 4) {
    dma_step<TRA, TRB, true, true, 2, true>(s3, s0, s1, acc, f0, f1, issue, issue, wm, cb0);
    dma_step<TRA, TRB, true, true, 2, true>(s0, s1, s2, acc, f0, f1, issue, issue, wm, cb0);
    dma_step<TRA, TRB, true, true, 2, true>(s1, s2, s3, acc, f0, f1, issue, issue, wm, cb0);
    dma_step<TRA, TRB, true, true, 2, true>(s2, s3, s0, acc, f0, f1, issue, issue, wm, cb0);
  }
  dma_step<TRA, TRB, true, false, 2, true>(s3, s0, s1, acc, f0, f1, issue, issue, wm, cb0);
  dma_step<TRA, TRB, false, false, 1, true>(s0, s1, s2, acc, f0, f1, issue, issue, wm, cb0);
  dma_step<TRA, TRB, false, false, 0, true>(s1, s2, s3, acc, f0, f1, issue, issue, wm, cb0);
  dma_step<TRA, TRB, false, false, 0, false>(s2, s3, s0, acc, f0, f1, issue, issue, wm, cb0);
  __syncthreads();                                     // all waves done with the last tile: LDS is free
}

// The K loop of a workgroup that goes on to another output tile afterwards (persistent kernels).
// On entry K tiles 0, 1, 2 of `issue` have been issued into s0, s1, s2 (dma_prefetch3, or the previous
// call of this function) and nothing of tile 3.  The last four steps, which have nothing left to fetch
// for this output tile, issue K tiles 0, 1, 2 of `next`, the sequence of the workgroup's next output
// tile, into the stages as they fall free: the pipeline never drains between output tiles, and stage s3
// -- free for every wave once it is past the last step's barrier -- is where the epilogue puts its
// patches.  There is one code path only (two, chosen by a branch, make the compiler shuffle the
// accumulator registers where they join): a workgroup on its last tile passes a sequence whose loads
// are valid but never used, and waits for them before it ends.  Global
// stores of the previous epilogue may still be in flight on entry: they only make the hand-placed
// wait counts conservative (a wait for "at most n operations in flight" covers every load that has n
// younger loads, whatever else is in the queue).  after_barrier() runs once behind the first barrier,
// when every wave has left the previous epilogue.
template <typename Issue> __device__ __forceinline__ void dma_prefetch3(lds_byte_t* s0, lds_byte_t* s1, lds_byte_t* s2, Issue& issue) {
  lds_byte_t* const stages[3] = {s0, s1, s2};
#pragma unroll
  for (int t = 0; t < 3; ++t) {
    issue.begin();
#pragma unroll
    for (int q = 0; q < 2 * kOpLoads; ++q) issue.part(stages[t], q);
    issue.end();
  }
}
// make_next(next) builds the next tile's sequence; it is called behind the steady-state loop, so that the
// sequence's registers are not live across it (spilled registers come back through the same in-order
// queue as the operand tiles: every reload inside the K loop would wait for all tiles in flight).
template <bool TRA, bool TRB, typename Issue, typename After, typename MakeNext>
__device__ __forceinline__ void dma_pipeline_cont(lds_byte_t* s0, lds_byte_t* s1, lds_byte_t* s2, lds_byte_t* s3,
                                                  DmaAcc& acc, Issue& issue, int KT, Issue& next, int wm,
                                                  int cb0, After after_barrier, MakeNext make_next) {
  wait_tiles_in_flight<2>();                           // tile 0 has landed
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
  issue.begin();
#pragma unroll
  for (int q = 0; q < kOpLoads; ++q) issue.part(s3, q);       // tile 3: first half
  after_barrier();
  DmaFrags f0, f1;
  dma_read_frags<TRA, TRB>(f0, s0, 0, wm, cb0);
  for (int kt = 0; kt < KT - 4; kt += 4) {
    dma_step<TRA, TRB, true, true, 2, true>(s3, s0, s1, acc, f0, f1, issue, issue, wm, cb0);
    dma_step<TRA, TRB, true, true, 2, true>(s0, s1, s2, acc, f0, f1, issue, issue, wm, cb0);
    dma_step<TRA, TRB, true, true, 2, true>(s1, s2, s3, acc, f0, f1, issue, issue, wm, cb0);
    dma_step<TRA, TRB, true, true, 2, true>(s2, s3, s0, acc, f0, f1, issue, issue, wm, cb0);
  }
  make_next(next);
  dma_step<TRA, TRB, true, true, 2, true>(s3, s0, s1, acc, f0, f1, issue, next, wm, cb0);
  dma_step<TRA, TRB, true, true, 2, true>(s0, s1, s2, acc, f0, f1, next, next, wm, cb0);
  dma_step<TRA, TRB, true, true, 2, true>(s1, s2, s3, acc, f0, f1, next, next, wm, cb0);
  dma_step<TRA, TRB, true, false, 0, false>(s2, s3, s0, acc, f0, f1, next, next, wm, cb0);
}

// Arguments of one rows GEMM (device pointers; see rows_gemm_persist_bf16).
struct RowsDmaArgs {
  const bf16_t* in;
  const bf16_t* w;
  const bf16_t* bias;
  const int32_t* voff;
  const int32_t* owner;
  int V, K, NC, row_tiles_max, col_tiles;
  const bf16_t* hpre_in;
  bf16_t* out0;
  bf16_t* out1;
  const int32_t* gsrc;
  int gk;
  float* split_partial;      // fp32 partial tiles of split tail tiles, or null: no splitting
  unsigned normal_grid;      // blocks before the extra segment workgroups (meaningful with split_partial)
  const int32_t* scatter_rows;   // plain epilogue only: bucket row p is stored as output row scatter_rows[p]; or null
};

// Sum of the K segments of the split tail tiles (see lookup_row_tile): out = bf16(sum over
// segments in order + bias).  Grid: (kSplitSlices row slices of a tile, kSplitUnits / 2 tail tiles at most).
constexpr int kSplitSlices = 16;
__global__ __launch_bounds__(kGemmThreads) void rows_split_reduce_kernel(const RowsDmaArgs p) {
  __shared__ int s_tile[8];
  RowTile t;
  const SplitArg sp{p.normal_grid, p.K / DK, (int)blockIdx.y};
  if (!lookup_row_tile<true>(p.voff, p.owner, p.V, p.NC, p.row_tiles_max, p.col_tiles, 0u, s_tile, &t, sp)) return;
  const float* part = p.split_partial + (size_t)(t.slot - t.seg) * (BM * BN);     // slot of segment 0
  constexpr int kRows = BM / kSplitSlices;                                        // rows per block
  constexpr int kIters = kRows * (BN / 4) / kGemmThreads;
  const int r0 = blockIdx.x * kRows;
  if (r0 >= t.rows_valid) return;
  float4 v[kIters][kSplitMax];
#pragma unroll
  for (int it = 0; it < kIters; ++it) {
    const int i4 = it * kGemmThreads + threadIdx.x;
    const int off = (r0 + i4 / (BN / 4)) * BN + (i4 % (BN / 4)) * 4;
#pragma unroll
    for (int sg = 0; sg < kSplitMax; ++sg)
      if (sg < t.nseg) v[it][sg] = *(const float4*)(part + (size_t)sg * (BM * BN) + off);
  }
#pragma unroll
  for (int it = 0; it < kIters; ++it) {
    const int i4 = it * kGemmThreads + threadIdx.x;
    const int row = r0 + i4 / (BN / 4), col = (i4 % (BN / 4)) * 4;
    float4 acc = v[it][0];
#pragma unroll
    for (int sg = 1; sg < kSplitMax; ++sg)
      if (sg < t.nseg) {
        acc.x += v[it][sg].x; acc.y += v[it][sg].y; acc.z += v[it][sg].z; acc.w += v[it][sg].w;
      }
    if (row < t.rows_valid && col < t.cols_valid) {
      if (p.bias) {
        float b[4];
        unpack4(*(const uint2*)(p.bias + (size_t)t.e * p.NC + t.n0 + col), b);
        acc.x += b[0]; acc.y += b[1]; acc.z += b[2]; acc.w += b[3];
      }
      const size_t orow = p.scatter_rows ? (size_t)p.scatter_rows[t.row0 + row] : (size_t)(t.row0 + row);
      *(uint2*)(p.out0 + orow * p.NC + t.n0 + col) = pack4(acc.x, acc.y, acc.z, acc.w);
    }
  }
}

}  // namespace flexmoe
