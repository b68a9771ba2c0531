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
// (16-byte chunk index XOR (row>>1)&3) is applied by choosing which global chunk a lane fetches.
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

// (Measured with ds_read_b128 alone: lane L reading row L % 16, chunk L / 16 -- the fragment of the 16 x 16 x 32
// instruction -- runs at 118 bytes per clock and compute unit with (row >> 2) & 3, at 180 with (row >> 1) & 3, which is
// what a conflict-free read reaches.)
__device__ __forceinline__ int dma_swz(int row) { return (row >> 1) & 3; }
__device__ __forceinline__ int dma_off(int row, int c) { return row * (DK * 2) + ((c ^ dma_swz(row)) << 4); }

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
      const int c = (i & 3) ^ dma_swz(row);
      off[q] = (uint32_t)(min(row, rows_valid - 1) * ld + c * 8) * 2;      // bytes
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
      const int c = (i & 3) ^ dma_swz(row);
      off[q] = (uint32_t)(((size_t)(rows[min(row, rows_valid - 1)] / k) * ld + c * 8) * 2);      // bytes: the matrix is below 2 GB (host check)
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
    // (uniform base in scalar registers + the lane's 32-bit byte offset: half the address registers of a 64-bit
    // pointer per lane, and no 64-bit add per load)
    const bf16_t* g = base + k0;
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" FLEXMOE_DMA_CPOL ::"v"(off[q]), "s"(g), "s"(lds0 + q * 1024) : "memory");
  }
};

// Operand stored [K, ld] with the output index contiguous (the forward weights W_e [K, NC]): the
// 32 x 256 tile is copied to LDS as it lies in memory, one k-row = 512 bytes = 32 chunks, two
// k-rows per direct-load instruction, and transposed on the way out of LDS by ds_read_tr16_b64.
// Chunk index XOR (k & 3) << 2 XOR (k & 8) >> 2 keeps those transposing reads free of bank conflicts: a
// group of 16 lanes reads 32 bytes of four consecutive k-rows (512 bytes apart: 64 bytes apart after the first
// term), and the neighbouring group the same columns eight k-rows further (32 bytes aside by the second).  Columns
// past cols_valid are clamped to the last valid 8-column chunk.
typedef short s16x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ int dmat_chunk(int krow, int c) { return c ^ ((krow & 3) << 2) ^ ((krow & 8) >> 2); }

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
      off[q] = (uint32_t)(krow * ld + c * 8) * 2;      // bytes
    }
  }
  __device__ __forceinline__ void part(lds_byte_t* tile, int k0, int q) const {
    const unsigned w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const unsigned lds0 = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)tile) + w * (kOpLoads * 1024);
    const bf16_t* g = base + (size_t)k0 * ld;
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" FLEXMOE_DMA_CPOL ::"v"(off[q]), "s"(g), "s"(lds0 + q * 1024) : "memory");
  }
};

// MFMA fragment (v_mfma_f32_16x16x32_bf16: 8 consecutive k of output column n0 + lane % 16, k = 8 (lane / 16) ..)
// from a [32 k][256 n] tile.  ds_read_tr16_b64 works on groups of 16 lanes: lanes 4m..4m+3 of a group
// address 16 consecutive elements of row m (4 each) and lane i of the group receives column i of
// those four rows.  So lane L (group g = L/16, i = L%16) points at row k = 8 g + i/4 (+4 for the second read),
// columns n0 + 4 (i%4): byte k * 512 + 16 dmat_chunk(k, col / 8) + 2 (col % 8) of the tile.  With n0 = 16 m that is
//   [k * 512 + 8 (i & 1) + 16 ((i & 3) >> 1) + 32 x(k)]  XOR  32 (m & 7),  + 256 (m >> 3),
// x(k) = 2 (k & 3) ^ ((k >> 3) & 1): a lane constant, a constant of the fragment XORed in, a constant added.
// The kernels keep only the lane constant in a register and form each fragment's address where it is read
// (kept per fragment, a dozen address registers would push the accumulators' neighbours into scratch).
__device__ __forceinline__ uint32_t dmat_lane(int L) {
  const int g = L >> 4, i = L & 15;
  const int k = 8 * g + (i >> 2);
  const int x = (((i >> 2) & 3) << 1) ^ (g & 1);
  return (uint32_t)(k * 512 + 8 * (i & 1) + 16 * ((i & 3) >> 1) + (x << 5));
}
__device__ __forceinline__ bf16x8 dmat_read_frag(const lds_byte_t* at) {
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)at);
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(at + 4 * 512));
  typedef short s16x8 __attribute__((ext_vector_type(8)));
  const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, v);
}
// The same for a [256][32 k] tile (dma_off): lane L reads the 16 bytes of row n0 + L % 16, chunk L / 16; n0 = 16 m
// only adds 1024 m.
__device__ __forceinline__ uint32_t dma_lane(int L) { return (uint32_t)dma_off(L & 15, L >> 4); }

// s_waitcnt vmcnt(n) only (expcnt / lgkmcnt fields left at "no wait").
template <int N> __device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit field");
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}
// Returns once at most `tiles` of the most recently issued K tiles (2 kOpLoads direct loads per wave each) are in flight.
template <int TILES> __device__ __forceinline__ void wait_tiles_in_flight() { wait_vmcnt<2 * kOpLoads * TILES>(); }

// The matrix instruction is v_mfma_f32_16x16x32_bf16: on real operands the chip holds a higher clock with it than
// with the 32 x 32 x 16 form (half the accumulator traffic per flop; the instruction alone: 2.13 against 1.94 PFLOP/s).
// A wave's 128 x 64 block is 8 x 4 of its 16 x 16 tiles.  Called as (column fragment, row fragment), lane L of a
// tile holds row L % 16 and the four consecutive columns 4 (L / 16) ..: acc[i][j][2 si + sj] is the tile of rows
// 16 si .., columns 16 sj .. of the wave's 32-row block i and 32-column block j.
typedef f32x16 DmaAcc[MB][NBW];      // [i][j], elements 4 (2 si + sj) .. + 3: one 16 x 16 tile each
__device__ __forceinline__ void zero_acc(DmaAcc& acc) {
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NBW; ++j)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.f;
}
// A K tile is multiplied in two halves: row blocks 0, 1 of the wave (a0: four 16-row fragments), then 2, 3 (a1),
// each against all four 16-column fragments b, which are read once per tile.
struct DmaFrags {
  Frag8 a0[4], a1[4], b[4];
  uint32_t la, lb;      // lane parts of the fragment addresses inside a stage (first / second operand)
};
// TRA / TRB: the operand's LDS tile is [k][256] (transposing reads) instead of [256][k].
template <bool TRA, bool TRB> __device__ __forceinline__ void dma_lane_init(DmaFrags& f, int wm, int cb0) {
  const int L = opaque_tid() & 63;
  f.la = TRA ? dmat_lane(L) ^ (uint32_t)(wm << 6) : dma_lane(L) + wm * 2048;
  f.lb = kDmaTileBytes + (TRB ? (dmat_lane(L) ^ (uint32_t)(((2 * cb0) & 4) << 5)) + (cb0 >> 2) * 256 : dma_lane(L) + cb0 * 2048);
}
// The four row fragments of half `half` (row blocks i = 2 half, 2 half + 1 of the wave, rows 16 si .. of each;
// 16-row unit m = 2 wm + 4 i + si, la carries the wave's wm).
template <bool TR> __device__ __forceinline__ void dma_read_rows(Frag8 (&a)[4], const lds_byte_t* stage, uint32_t la, int half) {
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    const int i = 2 * half + (p >> 1), si = p & 1;
    if (TR) a[p].v = dmat_read_frag(stage + ((la ^ (uint32_t)((4 * (i & 1) + si) << 5)) + (i >> 1) * 256));
    else a[p].v = *(const __attribute__((address_space(3))) bf16x8*)(stage + (la + i * 4096 + si * 1024));
  }
}
// Column fragment q (columns 32 (cb0 + q / 2) + 16 (q % 2) ..) of the second operand's tile (lb carries cb0 and
// the tile's place in the stage).
template <bool TR> __device__ __forceinline__ void dma_read_col(Frag8& b, const lds_byte_t* stage, uint32_t lb, int q) {
  if (TR) b.v = dmat_read_frag(stage + (lb ^ (uint32_t)(q << 5)));
  else b.v = *(const __attribute__((address_space(3))) bf16x8*)(stage + (lb + (q >> 1) * 2048 + (q & 1) * 1024));
}
// Everything the first half of a tile's step needs (the K loop's entry).
template <bool TRA, bool TRB>
__device__ __forceinline__ void dma_read_first(DmaFrags& f, const lds_byte_t* stage, int wm, int cb0) {
  dma_lane_init<TRA, TRB>(f, wm, cb0);
  dma_read_rows<TRA>(f.a0, stage, f.la, 0);
#pragma unroll
  for (int q = 0; q < 4; ++q) dma_read_col<TRB>(f.b[q], stage, f.lb, q);
}
// The 16 matrix instructions of column fragment q against the four row fragments of half `half`.
// PRIO: the wave runs its four instructions at raised priority (the SIMD's other wave then gets its loads and LDS
// reads in behind them instead of between them).  Measured on the GPT-XL-like layer: backward products -0.4 ... -0.7 %,
// forward products (one operand read with transposing loads) +0.3 %, so only the former ask for it.
template <bool PRIO>
__device__ __forceinline__ void dma_mfma_group(DmaAcc& acc, const Frag8 (&a)[4], const Frag8& b, int half, int q) {
  if (PRIO) __builtin_amdgcn_s_setprio(1);
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    f32x16& t = acc[2 * half + (p >> 1)][q >> 1];
    const int e = 4 * (2 * (p & 1) + (q & 1));
    f32x4 c = {t[e], t[e + 1], t[e + 2], t[e + 3]};
    c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b.v, a[p].v, c, 0, 0, 0);
    t[e] = c[0];
    t[e + 1] = c[1];
    t[e + 2] = c[2];
    t[e + 3] = c[3];
  }
  if (PRIO) __builtin_amdgcn_s_setprio(0);
}

// One K tile.  On entry f.a0 and f.b hold the fragments of tile kt's first half.
// The barrier sits between the two halves: before it the wave has fetched everything it needs
// from `cur`, so after it `cur` is free for tile kt+4; and tile kt+1 is published, so its first
// fragments can be fetched while the second half's MFMAs run -- no LDS latency after the barrier: the row
// fragments at once (a0 is free), each column fragment as soon as the second half is done with the current one.
// The direct loads are spread evenly between the MFMAs, one after every eight (128 cycles of
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
                                         DmaFrags& f, Issue& issue, IssuePost& issue_post, int wm, int cb0) {
  constexpr int kEvery = 4 / kOpLoads;      // a load after every kEvery-th group of four MFMAs
  // (behind an empty asm: each fragment address is derived from these where it is used, not once for the whole loop)
  asm volatile("" : "+v"(f.la), "+v"(f.lb));
  const uint32_t la = f.la, lb = f.lb;
  dma_read_rows<TRA>(f.a1, cur, la, 1);
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    __builtin_amdgcn_sched_barrier(0);
    dma_mfma_group<TRA == TRB>(acc, f.a0, f.b[q], 0, q);
    __builtin_amdgcn_sched_barrier(0);
    if (PRE && q % kEvery == kEvery - 1) issue.part(prev, kOpLoads + q / kEvery);
  }
  if (PRE) issue.end();
  __builtin_amdgcn_sched_barrier(0);     // everything above is queued before the wave goes to wait
  if (NEXT) wait_tiles_in_flight<WAIT>();
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
  if (NEXT) dma_read_rows<TRA>(f.a0, nxt, la, 0);
  if (POST) issue_post.begin();
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    __builtin_amdgcn_sched_barrier(0);
    dma_mfma_group<TRA == TRB>(acc, f.a1, f.b[q], 1, q);
    if (NEXT) dma_read_col<TRB>(f.b[q], nxt, lb, q);
    __builtin_amdgcn_sched_barrier(0);
    if (POST && q % kEvery == kEvery - 1) issue_post.part(cur, q / kEvery);
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
  DmaFrags f;
  dma_read_first<TRA, TRB>(f, s0, wm, cb0);
  for (int kt = 0; kt < KT - 4; kt += 4) {
    dma_step<TRA, TRB, true, true, 2, true>(s3, s0, s1, acc, f, issue, issue, wm, cb0);
    dma_step<TRA, TRB, true, true, 2, true>(s0, s1, s2, acc, f, issue, issue, wm, cb0);
    dma_step<TRA, TRB, true, true, 2, true>(s1, s2, s3, acc, f, issue, issue, wm, cb0);
    dma_step<TRA, TRB, true, true, 2, true>(s2, s3, s0, acc, f, issue, issue, wm, cb0);
  }
  dma_step<TRA, TRB, true, false, 2, true>(s3, s0, s1, acc, f, issue, issue, wm, cb0);
  dma_step<TRA, TRB, false, false, 1, true>(s0, s1, s2, acc, f, issue, issue, wm, cb0);
  dma_step<TRA, TRB, false, false, 0, true>(s1, s2, s3, acc, f, issue, issue, wm, cb0);
  dma_step<TRA, TRB, false, false, 0, false>(s2, s3, s0, acc, f, issue, issue, wm, cb0);
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
  DmaFrags f;
  dma_read_first<TRA, TRB>(f, s0, wm, cb0);
  for (int kt = 0; kt < KT - 4; kt += 4) {
    dma_step<TRA, TRB, true, true, 2, true>(s3, s0, s1, acc, f, issue, issue, wm, cb0);
    dma_step<TRA, TRB, true, true, 2, true>(s0, s1, s2, acc, f, issue, issue, wm, cb0);
    dma_step<TRA, TRB, true, true, 2, true>(s1, s2, s3, acc, f, issue, issue, wm, cb0);
    dma_step<TRA, TRB, true, true, 2, true>(s2, s3, s0, acc, f, issue, issue, wm, cb0);
  }
  make_next(next);
  dma_step<TRA, TRB, true, true, 2, true>(s3, s0, s1, acc, f, issue, next, wm, cb0);
  dma_step<TRA, TRB, true, true, 2, true>(s0, s1, s2, acc, f, next, next, wm, cb0);
  dma_step<TRA, TRB, true, true, 2, true>(s1, s2, s3, acc, f, next, next, wm, cb0);
  dma_step<TRA, TRB, true, false, 0, false>(s2, s3, s0, acc, f, next, next, wm, cb0);
  __builtin_amdgcn_sched_barrier(0);      // the epilogue's preparations stay behind the last MFMAs (registers)
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
