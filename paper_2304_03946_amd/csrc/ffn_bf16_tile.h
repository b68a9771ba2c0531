// Tile mapping, register-staged operand loads, LDS -> MFMA fragments, activation tables, epilogues and the register-staged rows kernel.
// Part of the bf16 expert-FFN kernels; included by ffn_bf16.hip only (one translation unit).
#pragma once
#include "common.h"

namespace flexmoe {

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int kGemmThreads = 256;
constexpr int MB = 4, NB = 4;                       // 32x32 MFMA tiles per wave: 4 x 4
constexpr int kTileElems = BM * BK;                 // one operand tile in LDS (elements)
constexpr size_t kGemmLds = 2 * 2 * kTileElems * sizeof(bf16_t);   // 2 stages x (A + B) = 128 KB

enum { EPI_FWD1 = 0, EPI_PLAIN = 1, EPI_DH = 2, EPI_DHQ = 3 };      // DHQ: dH * act'(Hpre) only (H was kept by the forward)
#ifndef FLEXMOE_EPI_AHEAD
#define FLEXMOE_EPI_AHEAD 2      // rounds between the request and the use of an epilogue side input
#endif
#ifndef FLEXMOE_DMA_CPOL
#define FLEXMOE_DMA_CPOL ""      // cache-policy modifiers of the direct-to-LDS loads
#endif

// threadIdx.x behind a compiler barrier: what is derived from it is computed where it is used.  The
// persistent kernels use it for per-lane constants of code that runs once per output tile (operand
// offsets, epilogue addressing): taken from threadIdx.x directly they are loop invariants, which the
// compiler computes once, keeps across the K loop and, out of registers there, spills -- and a spilled
// register comes back through the queue the operand tiles are in flight in.
__device__ __forceinline__ int opaque_tid() {
  int t = threadIdx.x;
  asm volatile("" : "+v"(t));
  return t;
}

union Frag8 {
  uint4 u;
  bf16x8 v;
};

__device__ __forceinline__ int swz(int row) { return (row ^ (row >> 3)) & 7; }
__device__ __forceinline__ int lds_off(int row, int chunk) { return row * BK + ((chunk ^ swz(row)) << 3); }

// ---- workgroup id -> tile, XCD aware ---------------------------------------------------------
// Workgroups are dealt round-robin to the 8 XCDs (id % 8), each with its own L2, and an XCD runs
// its workgroups in ascending id.  The rows x cols tile grid is cut into column strips pw tiles wide
// (pw divides cols whenever a divisor in 5..8 exists) and every strip, walked row by row, into patches
// of 32 consecutive tiles (one per CU of an XCD: 32 / pw rows of the strip; where pw does not divide 32
// a patch starts and ends inside a row); the j-th workgroup of XCD x gets tile j % 32 of patch
// (j / 32) * 8 + x, patches numbered strip by strip within a row of patches.  The workgroups that run
// together on one XCD then share about 32 / pw row operands and pw column operands in its L2, and the 8
// patches in flight on the 8 XCDs are neighbours in the grid, so what they share is fetched from HBM once.
constexpr int kXcds = 8, kPatch = 32;
__host__ __device__ inline int patch_width(int cols) {
  if (cols <= 8) return cols;
  for (int pw = 8; pw >= 5; --pw)
    if (cols % pw == 0) return pw;
  return 8;
}
__host__ __device__ inline unsigned patched_grid(int rows, int cols) {
  const int pw = patch_width(cols);
  const int np = ((rows * pw + kPatch - 1) / kPatch) * ((cols + pw - 1) / pw);
  return (unsigned)((np + kXcds - 1) / kXcds * kXcds) * kPatch;
}
// returns false when the workgroup falls into the padding of the patch grid
__device__ __forceinline__ bool patched_tile(unsigned b, int rows, int cols, int* r, int* c) {
  const int pw = patch_width(cols);
  const int npc = (cols + pw - 1) / pw;
  const unsigned x = b % kXcds, j = b / kXcds;
  const unsigned P = (j / kPatch) * kXcds + x, q = j % kPatch;
  const unsigned t = (P / npc) * kPatch + q;      // position in the strip's row-by-row walk
  *r = (int)(t / pw);
  *c = (int)(P % npc) * pw + (int)(t % pw);
  return *r < rows && *c < cols;
}

// ---- global -> registers -> LDS -------------------------------------------------------------
// Workgroup barrier that orders LDS traffic only: global loads issued for a later tile stay in
// flight across it (a full __syncthreads would wait for them).
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Operand stored [rows, ld] with the contraction index contiguous.  Thread t owns 16-byte chunk
// t&7 of rows (t>>3) + 32*i.  Rows past rows_valid are clamped to the last valid row (their
// products are never stored), so full-K tiles load without predication; a ragged last K tile
// reads chunks past K as zero.
struct KContigSrc {
  const bf16_t* base;
  uint32_t off[8];
  int K;
  __device__ __forceinline__ void init(const bf16_t* b, size_t ld, int rows_valid, int K_) {
    base = b;
    K = K_;
    const int c = threadIdx.x & 7, rr = threadIdx.x >> 3;
#pragma unroll
    for (int i = 0; i < 8; ++i) off[i] = (uint32_t)(min(rr + 32 * i, rows_valid - 1) * ld + c * 8);
  }
  __device__ __forceinline__ void load(uint4 (&r)[8], int k0) const {
    if (k0 + BK <= K) {
#pragma unroll
      for (int i = 0; i < 8; ++i) r[i] = *(const uint4*)(base + k0 + off[i]);
    } else {
      const bool kok = k0 + (int)(threadIdx.x & 7) * 8 < K;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        r[i] = make_uint4(0, 0, 0, 0);
        if (kok) r[i] = *(const uint4*)(base + k0 + off[i]);
      }
    }
  }
  static __device__ __forceinline__ void store(bf16_t* tile, const uint4 (&r)[8]) {
    const int c = threadIdx.x & 7, rr = threadIdx.x >> 3;
#pragma unroll
    for (int i = 0; i < 8; ++i) *(uint4*)(tile + lds_off(rr + 32 * i, c)) = r[i];
  }
};

// Operand stored [K, ld] with the output index contiguous.  Thread t owns the 8x8 block at
// k = 8*(t>>5).., column 8*(t&31)..; columns past cols_valid are clamped to the last valid
// 8-column group; contraction rows >= k_valid read as zero (they would add to the sums).
struct KStridedSrc {
  uint32_t off[8];
  __device__ __forceinline__ void init(size_t ld, int cols_valid) {
    const int nc = min((int)(threadIdx.x & 31), cols_valid / 8 - 1), kc = threadIdx.x >> 5;
#pragma unroll
    for (int j = 0; j < 8; ++j) off[j] = (uint32_t)((kc * 8 + j) * ld + nc * 8);
  }
  // `p` points at contraction row 0 of this tile, first column of the tile
  __device__ __forceinline__ void load(uint4 (&r)[8], const bf16_t* __restrict__ p, int k_valid) const {
    if (k_valid >= BK) {
#pragma unroll
      for (int j = 0; j < 8; ++j) r[j] = *(const uint4*)(p + off[j]);
    } else {
      const int kc = threadIdx.x >> 5;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        r[j] = make_uint4(0, 0, 0, 0);
        if (kc * 8 + j < k_valid) r[j] = *(const uint4*)(p + off[j]);
      }
    }
  }
  static __device__ __forceinline__ uint32_t lo16(uint32_t a, uint32_t b) { return (a & 0xffffu) | (b << 16); }
  static __device__ __forceinline__ uint32_t hi16(uint32_t a, uint32_t b) { return (a >> 16) | (b & 0xffff0000u); }
  // r[j] holds columns 0..7 of k-row j; emit, per column n, its 8 k-values as one 16-byte chunk
  static __device__ __forceinline__ void store(bf16_t* tile, const uint4 (&r)[8]) {
    const int nc = threadIdx.x & 31, kc = threadIdx.x >> 5;
    uint4 o;
#define FLEXMOE_TR(n, comp, pick)                                                                    \
  o = make_uint4(pick(r[0].comp, r[1].comp), pick(r[2].comp, r[3].comp), pick(r[4].comp, r[5].comp), \
                 pick(r[6].comp, r[7].comp));                                                        \
  *(uint4*)(tile + lds_off(nc * 8 + n, kc)) = o;
    FLEXMOE_TR(0, x, lo16) FLEXMOE_TR(1, x, hi16) FLEXMOE_TR(2, y, lo16) FLEXMOE_TR(3, y, hi16)
    FLEXMOE_TR(4, z, lo16) FLEXMOE_TR(5, z, hi16) FLEXMOE_TR(6, w, lo16) FLEXMOE_TR(7, w, hi16)
#undef FLEXMOE_TR
  }
};

// ---- LDS -> MFMA ---------------------------------------------------------------------------
// One 16-wide k step of the wave's 128x128 block.
// acc[i][j]: output rows (wm + 2*i)*32 + lane%32, columns (wn*NB + j)*32 + 8*(q/4) + 4*(lane/32) + q%4.
template <bool FULL>
__device__ __forceinline__ void mma_kstep(const bf16_t* __restrict__ As, const bf16_t* __restrict__ Bs, int s,
                                          f32x16 (&acc)[MB][NB], int wm, int wn, int nblk_rows) {
  const int lane = threadIdx.x & 63;
  const int r = lane & 31, h = lane >> 5;
  Frag8 af[MB], bfr[NB];
#pragma unroll
  for (int i = 0; i < MB; ++i)
    if (FULL || wm + 2 * i < nblk_rows) af[i].u = *(const uint4*)(As + lds_off((wm + 2 * i) * 32 + r, 2 * s + h));
#pragma unroll
  for (int j = 0; j < NB; ++j) bfr[j].u = *(const uint4*)(Bs + lds_off((wn * NB + j) * 32 + r, 2 * s + h));
#pragma unroll
  for (int i = 0; i < MB; ++i)
    if (FULL || wm + 2 * i < nblk_rows) {
#pragma unroll
      for (int j = 0; j < NB; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j].v, af[i].v, acc[i][j], 0, 0, 0);
    }
}

__device__ __forceinline__ void zero_acc(f32x16 (&acc)[MB][NB]) {
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.f;
}

__device__ __forceinline__ uint2 pack4(float a, float b, float c, float d) {
  return make_uint2(pack_bf16x2(a, b), pack_bf16x2(c, d));
}
__device__ __forceinline__ void unpack4(uint2 u, float* v) {
  v[0] = __uint_as_float(u.x << 16);
  v[1] = __uint_as_float(u.x & 0xffff0000u);
  v[2] = __uint_as_float(u.y << 16);
  v[3] = __uint_as_float(u.y & 0xffff0000u);
}

// ---- activation tables -------------------------------------------------------------------------
// The GELU epilogues act on pre-activations already rounded to bf16, so the activation has only
// 2^16 possible arguments.  Both GELU forms are z*F(z) with F(z) + F(-z) = 1, which makes
//   GELU(z)  = max(z, 0) + r(|z|),          r(a) = GELU(a) - a   (= GELU(-a), even in z)
//   GELU'(z) = [z >= 0] + sign(z) * q(|z|),  q(a) = GELU'(a) - 1
// so one table over the bf16 magnitudes serves both signs.  r and q vanish (below 1e-13) from
// |z| = 8 on and r(a) -> -a/2, q -> -1/2 as a -> 0: magnitudes are clamped to [2^-24, 8], which
// costs an absolute error below 2^-25.  Entries are computed in double precision when the library is
// built (gen_act_lut.py writes act_lut_data.inc) and live in the code object as constant {r, q} fp32
// pairs: 3457 entries, padded to 28 KB so that the GEMM kernels can pull the table into LDS with
// whole 1 KB direct loads.  Nothing is filled in at run time: no first-call set-up, no host-side state.
constexpr int kLutLo = 103 << 7;                    // bf16 bits of 2^-24
constexpr int kLutHi = 130 << 7;                    // bf16 bits of 8.0
constexpr int kLutBytes = 28 * 1024;
constexpr int kLutEntries = kLutBytes / 8;
static_assert(kLutHi - kLutLo + 1 <= kLutEntries, "table does not fit its padding");
struct ActLutEntry {
  float r, q;
};
__device__ __align__(1024) const ActLutEntry g_act_lut[2][kLutEntries] = {      // [0] erf form, [1] tanh form
#include "act_lut_data.inc"
};
static_assert(sizeof(g_act_lut) == 2 * kLutBytes, "generated table and layout constants disagree");

// Table entry for the bf16 value whose fp32 bit pattern is zu (LDS copy of one table).
typedef __attribute__((address_space(3))) unsigned char lds_byte_t;
typedef __attribute__((address_space(3))) int lds_int_t;
__device__ __forceinline__ uint32_t lut_offset(uint32_t zu) {
  const uint32_t m = (zu >> 16) & 0x7fffu;
  return (min(max(m, (uint32_t)kLutLo), (uint32_t)kLutHi) - kLutLo) << 3;
}
// max(z, 0) on the bit pattern: as a signed integer every negative float (and -0) is below zero
// and every positive float keeps its order, so one integer max does it (no NaN canonicalisation).
__device__ __forceinline__ float relu_bits(uint32_t zu) { return __int_as_float(max((int32_t)zu, 0)); }
__device__ __forceinline__ float lut_act(const lds_byte_t* lut, uint32_t zu) {
  const float r = *(const __attribute__((address_space(3))) float*)(lut + lut_offset(zu));
  return relu_bits(zu) + r;
}
__device__ __forceinline__ void lut_act_both(const lds_byte_t* lut, uint32_t zu, float* a, float* da) {
  const f32x2_t rq = *(const __attribute__((address_space(3))) f32x2_t*)(lut + lut_offset(zu));
  *a = relu_bits(zu) + rq[0];
  *da = (int32_t)zu < 0 ? -rq[1] : 1.f + rq[1];
}
__device__ __forceinline__ float lut_act_d(const lds_byte_t* lut, uint32_t zu) {
  const float q = *(const __attribute__((address_space(3))) float*)(lut + lut_offset(zu) + 4);
  return (int32_t)zu < 0 ? -q : 1.f + q;
}
template <int EPI, int ACT> constexpr bool epilogue_uses_lut() { return EPI != EPI_PLAIN && ACT != FLEXMOE_RELU; }

// ---- epilogue ---------------------------------------------------------------------------------
// A lane's accumulators hold 4-column pieces of 32 different rows, which would make every global
// store touch 32 cache lines.  Instead the wave's 128x128 fp32 block goes out in eight rounds of
// 32 rows x 64 columns: accumulator registers -> one of two wave-private 8 KB LDS patches (16-byte chunks,
// chunk index XORed with row & 15: conflict free both ways) -> read back so that 16 lanes cover
// 64 consecutive columns of one row -> per-element epilogue in fp32 -> bf16 -> 8-byte stores that
// fill whole 128-byte lines.  The K loop ends with a barrier, so the LDS tiles are free.
// Per round, all eight 4-element pieces are first computed (compute(row in the wave's block
// (0..127), column in the wave's block (multiple of 4), which 64-column half of the block that is,
// float4 accumulators, uint2 side input) -> EpiOut, unconditional: straight-line code the scheduler
// can interleave) and then stored (store(row, col, EpiOut), where the ragged-edge predicates live).
// fetch(row, col) -> uint2: an optional per-element side input (the saved pre-activations of the
// backward epilogue).
struct EpiOut {
  uint2 a, b;
};
// Which 4-element piece a callback of epilogue_rounds is asked about: 32-row block i (0..MB-1) and 64-column
// half jh of the wave's 128 x 128 block, piece it (0..7) of the round -- compile-time constants once the
// loops are unrolled -- and the same as lane-dependent coordinates inside the wave's block:
// row_w = 32 i + 4 it + (lane / 16), col_w = 64 jh + 4 (lane % 16).
// (Eight-wave kernels, epilogue_rounds8: a wave owns one 64-column half, jh is then uniform over the wave, and a
// round covers 16 rows: sub = which half of the 32-row block, row_w = 32 i + 16 sub + 4 it + (lane / 16), it < 4.)
struct EpiIdx {
  int i, jh, it;
  int row_w, col_w;
  int sub;
};
// 8-byte store with the non-temporal hint.  Used for the large outputs of the epilogues that carry an
// activation (Hpre and H of the forward, dHpre and H of the backward) and for the weight gradients:
// streamed out, they do not displace the operands the running product keeps re-reading in L2 and the
// Infinity Cache (measured: -4.5 % on the BERT-like layer's step, -2.4 % on the GPT-medium-like one,
// -1 % on the GPT-XL-like one).  The plain epilogue's output (Yp, dXp) keeps the default policy: the
// combine kernel reads it straight away, and streaming it out costs there what it gains here.
__device__ __forceinline__ void store_nt8(void* p, uint2 v) {
  typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
  u32x2_t v2;
  v2[0] = v.x;
  v2[1] = v.y;
  __builtin_nontemporal_store(v2, (u32x2_t*)p);
}
template <bool FETCH, typename Fetch, typename Compute, typename Store>
__device__ __forceinline__ void epilogue_rounds(float* patch0, float* patch1, const f32x16 (&acc)[MB][NB], Fetch fetch,
                                                Compute compute, Store store) {
  const int lane = opaque_tid() & 63;
  const int r = lane & 31, h = lane >> 5;
  const int rsub = lane >> 4, c = lane & 15;
  constexpr int kRounds = MB * (NB / 2);
  auto idx_of = [&](int round, int it) {
    const int i = round / (NB / 2), jh = round % (NB / 2);
    return EpiIdx{i, jh, it, i * 32 + it * 4 + rsub, jh * 64 + c * 4, 0};
  };
  // Side inputs are requested kAhead rounds before they are used.  Loads and stores of a wave complete
  // in issue order: a load issued behind a round's stores only returns once those stores are
  // acknowledged, so a request made one round ahead puts a store round trip into every round.
  constexpr int kAhead = FLEXMOE_EPI_AHEAD;
  uint2 side[FETCH ? kAhead + 1 : 1][8];
  auto fetch_round = [&](int round) {
#pragma unroll
    for (int it = 0; it < 8; ++it) side[round % (kAhead + 1)][it] = fetch(idx_of(round, it));
  };
  if (FETCH) {
#pragma unroll
    for (int round = 0; round < kAhead; ++round) fetch_round(round);
  }
  // Two patches per wave (or one, used twice): round n+1's accumulators are written while round n is
  // processed.  A wave's LDS instructions execute in issue order, so the reads that follow the writes
  // need no wait, only a compiler barrier (the dependence runs across lanes, which the compiler cannot see).
  auto write_round = [&](int i, int jh, float* patch) {
#pragma unroll
    for (int jj = 0; jj < 2; ++jj)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int cc = jj * 8 + 2 * g + h;
        const f32x16& a = acc[i][jh * 2 + jj];
        *(float4*)(patch + r * 64 + ((cc ^ (r & 15)) << 2)) = make_float4(a[4 * g], a[4 * g + 1], a[4 * g + 2], a[4 * g + 3]);
      }
  };
  write_round(0, 0, patch0);
#pragma unroll
  for (int round = 0; round < kRounds; ++round) {
    float* patch = (round & 1) ? patch1 : patch0;
    if (FETCH && round + kAhead < kRounds) fetch_round(round + kAhead);
    asm volatile("" ::: "memory");
    float4 v[8];
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const int row = it * 4 + rsub;
      v[it] = *(const float4*)(patch + row * 64 + ((c ^ (row & 15)) << 2));
    }
    asm volatile("" ::: "memory");
    if (round + 1 < kRounds) write_round((round + 1) / (NB / 2), (round + 1) % (NB / 2), (round & 1) ? patch0 : patch1);
    asm volatile("" ::: "memory");
    EpiOut o[8];
#pragma unroll
    for (int it = 0; it < 8; ++it)
      o[it] = compute(idx_of(round, it), v[it], FETCH ? side[round % (kAhead + 1)][it] : make_uint2(0, 0));
#pragma unroll
    for (int it = 0; it < 8; ++it) store(idx_of(round, it), o[it]);
  }
}

// The same for a wave of the eight-wave kernels: its accumulators are acc[i][0..1], the 64-column half jh of a
// 128-column block, and its patch holds 16 rows x 64 columns (4 KB: eight of them fit the one LDS stage a
// persistent kernel has free while its next tile's operands are landing in the others).  Eight rounds -- 32-row
// block i, rows 16 sub .. 16 sub + 15 of it: the four 16 x 16 accumulator tiles of those rows -- of four
// 4-element pieces per lane.
template <bool FETCH, typename Fetch, typename Compute, typename Store>
__device__ __forceinline__ void epilogue_rounds8(float* patch, int jh, const f32x16 (&acc)[MB][2], Fetch fetch,
                                                 Compute compute, Store store) {
  const int lane = opaque_tid() & 63;
  const int rsub = lane >> 4, c = lane & 15;
  constexpr int kRounds = MB * 2, kIts = 4;
  auto idx_of = [&](int round, int it) {
    const int i = round >> 1, sub = round & 1;
    return EpiIdx{i, jh, it, i * 32 + sub * 16 + it * 4 + rsub, jh * 64 + c * 4, sub};
  };
  constexpr int kAhead = FLEXMOE_EPI_AHEAD;
  uint2 side[FETCH ? kAhead + 1 : 1][kIts];
  auto fetch_round = [&](int round) {
#pragma unroll
    for (int it = 0; it < kIts; ++it) side[round % (kAhead + 1)][it] = fetch(idx_of(round, it));
  };
  if (FETCH) {
#pragma unroll
    for (int round = 0; round < kAhead; ++round) fetch_round(round);
  }
  // a round's write follows the previous round's reads in the wave's instruction stream: LDS executes a
  // wave's instructions in order, so one patch serves every round
  // (accumulator tile: elements 4 (2 sub + sj) .. of acc[i][jj]; the lane's row is lane % 16 of the round's 16, its four columns start at
  // 32 jj + 16 sj + 4 (lane / 16) of the wave's 64)
  auto write_round = [&](int i, int sub) {
#pragma unroll
    for (int jj = 0; jj < 2; ++jj)
#pragma unroll
      for (int sj = 0; sj < 2; ++sj) {
        const int cc = jj * 8 + sj * 4 + rsub;
        const f32x16& a = acc[i][jj];
        const int e = 4 * (2 * sub + sj);
        *(float4*)(patch + c * 64 + ((cc ^ c) << 2)) = make_float4(a[e], a[e + 1], a[e + 2], a[e + 3]);
      }
  };
  write_round(0, 0);
#pragma unroll
  for (int round = 0; round < kRounds; ++round) {
    if (FETCH && round + kAhead < kRounds) fetch_round(round + kAhead);
    asm volatile("" ::: "memory");
    float4 v[kIts];
#pragma unroll
    for (int it = 0; it < kIts; ++it) {
      const int row = it * 4 + rsub;
      v[it] = *(const float4*)(patch + row * 64 + ((c ^ row) << 2));
    }
    asm volatile("" ::: "memory");
    if (round + 1 < kRounds) write_round((round + 1) >> 1, (round + 1) & 1);
    asm volatile("" ::: "memory");
    EpiOut o[kIts];
#pragma unroll
    for (int it = 0; it < kIts; ++it)
      o[it] = compute(idx_of(round, it), v[it], FETCH ? side[round % (kAhead + 1)][it] : make_uint2(0, 0));
#pragma unroll
    for (int it = 0; it < kIts; ++it) store(idx_of(round, it), o[it]);
  }
}

// Addresses of the pieces of epilogue_rounds inside an output (or side input) tile whose rows are ld
// elements of ELEM bytes apart: piece (i, jh, it) is at [uniform: first element of 32-row block i,
// 64-column half jh of the wave's block] + [per lane, per it: byte offset of tile row wm*32 + 4 it +
// lane/16, column 4 (lane%16)].  The eight lane offsets are computed once per tile and the uniform part
// lives in scalar registers, so a store or load costs no address arithmetic.
template <int ELEM> struct EpiAddr {
  uint32_t vb[8];
  int ld;
  __device__ __forceinline__ void init(int wm, int ld_) {
    ld = ld_;
    const int lane = opaque_tid() & 63;
    const int rsub = lane >> 4, c = lane & 15;
#pragma unroll
    for (int it = 0; it < 8; ++it) vb[it] = (uint32_t)(((wm * 32 + it * 4 + rsub) * ld + c * 4) * ELEM);
  }
  // block_base: the wave's block of the tile (tile row 0, the wave's first column)
  template <typename T> __device__ __forceinline__ T* at(T* block_base, const EpiIdx& x) const {
    T* round_base = block_base + (size_t)(x.i * 64 + x.sub * 16) * ld + x.jh * 64;
    return (T*)((char*)round_base + vb[x.it]);
  }
};

// One K tile of the software pipeline.  On entry LDS stage `cur` holds tile t and the registers
// ra/rb hold tile t+1 (loaded during the previous step).  The tile is multiplied in four k
// steps; early in the step each register set is written to stage `nxt` and immediately reused
// for the loads of tile t+2, which then have most of a step of MFMA work to land.
template <bool FULL, bool STORE, bool LOAD, typename StoreA, typename StoreB, typename LoadA, typename LoadB>
__device__ __forceinline__ void pipe_step(bf16_t* cur, bf16_t* nxt, f32x16 (&acc)[MB][NB], uint4 (&ra)[8],
                                          uint4 (&rb)[8], StoreA store_a, StoreB store_b, LoadA& load_a, LoadB& load_b,
                                          int wm, int wn, int nblk_rows) {
  mma_kstep<FULL>(cur, cur + kTileElems, 0, acc, wm, wn, nblk_rows);
  if (STORE) store_a(nxt, ra);
  if (LOAD) load_a(ra);
  mma_kstep<FULL>(cur, cur + kTileElems, 1, acc, wm, wn, nblk_rows);
  if (STORE) store_b(nxt + kTileElems, rb);
  if (LOAD) load_b(rb);
  mma_kstep<FULL>(cur, cur + kTileElems, 2, acc, wm, wn, nblk_rows);
  mma_kstep<FULL>(cur, cur + kTileElems, 3, acc, wm, wn, nblk_rows);
  lds_barrier();
}

// Drives T tiles through the pipeline.  load_a(ra) / load_b(rb) fetch the next tile in sequence.
template <bool FULL, typename StoreA, typename StoreB, typename LoadA, typename LoadB>
__device__ __forceinline__ void run_pipeline(bf16_t* smem, f32x16 (&acc)[MB][NB], int T, StoreA store_a,
                                             StoreB store_b, LoadA& load_a, LoadB& load_b, int wm, int wn,
                                             int nblk_rows) {
  uint4 ra[8], rb[8];
  load_a(ra);
  load_b(rb);
  store_a(smem, ra);
  store_b(smem + kTileElems, rb);
  if (T > 1) {
    load_a(ra);
    load_b(rb);
  }
  lds_barrier();
  int t = 0;
  for (; t + 2 < T; ++t) {
    bf16_t* cur = smem + (t & 1) * 2 * kTileElems;
    bf16_t* nxt = smem + ((t & 1) ^ 1) * 2 * kTileElems;
    pipe_step<FULL, true, true>(cur, nxt, acc, ra, rb, store_a, store_b, load_a, load_b, wm, wn, nblk_rows);
  }
  if (t + 1 < T) {
    bf16_t* cur = smem + (t & 1) * 2 * kTileElems;
    bf16_t* nxt = smem + ((t & 1) ^ 1) * 2 * kTileElems;
    pipe_step<FULL, true, false>(cur, nxt, acc, ra, rb, store_a, store_b, load_a, load_b, wm, wn, nblk_rows);
    ++t;
  }
  {
    bf16_t* cur = smem + (t & 1) * 2 * kTileElems;
    pipe_step<FULL, false, false>(cur, cur, acc, ra, rb, store_a, store_b, load_a, load_b, wm, wn, nblk_rows);
  }
}

// K loop of rows_gemm.
template <bool WT, bool FULL>
__device__ __forceinline__ void rows_mainloop(bf16_t* smem, f32x16 (&acc)[MB][NB], const bf16_t* __restrict__ a_base,
                                              const bf16_t* __restrict__ w_e, int K, int NC, int n0, int rows_valid,
                                              int cols_valid, int wm, int wn, int nblk_rows) {
  const int KT = (K + BK - 1) / BK;
  KContigSrc a_src;
  a_src.init(a_base, K, rows_valid, K);
  int ka = 0, kb = 0;
  auto load_a = [&](uint4 (&ra)[8]) {
    a_src.load(ra, ka);
    ka += BK;
  };
  if (WT) {
    KContigSrc w_src;
    w_src.init(w_e + (size_t)n0 * K, K, cols_valid, K);
    auto load_b = [&](uint4 (&rb)[8]) {
      w_src.load(rb, kb);
      kb += BK;
    };
    run_pipeline<FULL>(smem, acc, KT, KContigSrc::store, KContigSrc::store, load_a, load_b, wm, wn, nblk_rows);
  } else {
    KStridedSrc w_src;
    w_src.init(NC, cols_valid);
    const bf16_t* wp = w_e + n0;
    auto load_b = [&](uint4 (&rb)[8]) {
      w_src.load(rb, wp + (size_t)kb * NC, K - kb);
      kb += BK;
    };
    run_pipeline<FULL>(smem, acc, KT, KContigSrc::store, KStridedSrc::store, load_a, load_b, wm, wn, nblk_rows);
  }
}

// Epilogue of the rows kernels: bias, then plain store / pre-activation + activation / dH*act' + H.
// LUT: the activation comes from the LDS copy `lut` of the activation table ({r, q} pairs, see
// above); otherwise it is evaluated arithmetically.
// FULL: all 256 rows of the tile and all 128 columns of the wave's block exist (no store predicates).
// SCATTER (plain epilogue): tile row r is stored as row smap[r] of out0.
// NW = 8: a wave of the eight-wave kernels (accumulators [MB][2], patches of 4 KB per wave at `lds`, lds_alt unused).
template <int EPI, int ACT, bool LUT, bool BIAS, bool FULL, bool SCATTER, int NW, typename Acc>
__device__ __forceinline__ void rows_epilogue_t(float* lds, float* lds_alt, const Acc& acc, const bf16_t* __restrict__ bias,
                                                int NC, int row0, int rows_valid, int e, int n0,
                                                const bf16_t* __restrict__ hpre_in, bf16_t* __restrict__ out0,
                                                bf16_t* __restrict__ out1, const lds_byte_t* lut,
                                                const lds_int_t* smap) {
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = (wave >> 1) & 1, wn = wave & 1, hh = wave >> 2;      // hh: the wave's 64-column half (eight waves)
  float* patch = lds + wave * (NW == 8 ? 16 * 64 : 32 * 64);
  float* patch_alt = lds_alt + wave * (32 * 64);
  const int col_base = n0 + wn * (NB * 32);
  // uniform per-tile base pointers (scalar registers) + per-lane 32-bit offsets
  const size_t tile_base = (size_t)row0 * NC + col_base;
  const bf16_t* hpre_t = hpre_in + tile_base;
  bf16_t* out0_t = out0 + tile_base;
  bf16_t* out1_t = out1 + tile_base;
  const bf16_t* bias_t = bias + (size_t)e * NC + col_base;
  const int cols_left = NC - col_base;
  EpiAddr<2> addr;
  addr.init(wm, NC);
  auto valid = [&](const EpiIdx& x) {
    return FULL || ((wm + 2 * x.i) * 32 + (x.row_w & 31) < rows_valid && x.col_w < cols_left);
  };
  auto fetch = [&](const EpiIdx& x) -> uint2 {
    if (valid(x)) return *(const uint2*)addr.at(hpre_t, x);
    return make_uint2(0, 0);
  };
  // the lane's bias values (two 64-column halves of the wave's block), read before any store is
  // issued: a load behind stores returns only once they are acknowledged
  float bvals[NB / 2][4];
  if (BIAS) {
    const int c4 = (opaque_tid() & 15) * 4;
#pragma unroll
    for (int jh = 0; jh < NB / 2; ++jh)      // eight waves: entry 0 holds the wave's own half
      unpack4(*(const uint2*)(bias_t + min((NW == 8 ? hh : jh) * 64 + c4, cols_left - 4)), bvals[jh]);
  }
  auto compute = [&](const EpiIdx& x, float4 c, uint2 pre_in) -> EpiOut {
    EpiOut o;
    if (BIAS) {
      const float* bv = bvals[NW == 8 ? 0 : x.jh];
      c.x += bv[0]; c.y += bv[1]; c.z += bv[2]; c.w += bv[3];
    }
    if (EPI == EPI_PLAIN) {
      o.a = pack4(c.x, c.y, c.z, c.w);
      o.b = make_uint2(0, 0);
    } else if (EPI == EPI_FWD1) {
      // keep the pre-activation; the activation is taken of the value as stored
      o.a = pack4(c.x, c.y, c.z, c.w);
      float z[4], a[4];
      unpack4(o.a, z);
#pragma unroll
      for (int q = 0; q < 4; ++q) a[q] = LUT ? lut_act(lut, __float_as_uint(z[q])) : act_fast<ACT>(z[q]);
      o.b = pack4(a[0], a[1], a[2], a[3]);
    } else if (EPI == EPI_DHQ) {
      float z[4], a, d[4];
      unpack4(pre_in, z);
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if (LUT) d[q] = lut_act_d(lut, __float_as_uint(z[q]));
        else act_both<ACT>(z[q], &a, &d[q]);
      }
      o.a = pack4(c.x * d[0], c.y * d[1], c.z * d[2], c.w * d[3]);
      o.b = make_uint2(0, 0);
    } else {
      float z[4], a[4], d[4];
      unpack4(pre_in, z);
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if (LUT) lut_act_both(lut, __float_as_uint(z[q]), &a[q], &d[q]);
        else act_both<ACT>(z[q], &a[q], &d[q]);
      }
      o.a = pack4(c.x * d[0], c.y * d[1], c.z * d[2], c.w * d[3]);
      o.b = pack4(a[0], a[1], a[2], a[3]);
    }
    return o;
  };
  const bool store0 = EPI != EPI_FWD1 || out0 != nullptr;      // forward: the pre-activations are optional
  auto store = [&](const EpiIdx& x, const EpiOut& o) {
    if (valid(x)) {
      if (SCATTER) {
        // scattered store: tile row lrow is row smap[lrow] of the output (reverse routing of a top-1 layer)
        const int lrow = (wm + 2 * x.i) * 32 + (x.row_w & 31);
        *(uint2*)(out0 + (size_t)smap[lrow] * NC + col_base + x.col_w) = o.a;
      } else if (store0) {
        if (EPI == EPI_PLAIN) *(uint2*)addr.at(out0_t, x) = o.a;
        else store_nt8(addr.at(out0_t, x), o.a);
      }
      if (EPI == EPI_FWD1 || EPI == EPI_DH) store_nt8(addr.at(out1_t, x), o.b);
    }
  };
  if constexpr (NW == 8) epilogue_rounds8<EPI == EPI_DH || EPI == EPI_DHQ>(patch, hh, acc, fetch, compute, store);
  else epilogue_rounds<EPI == EPI_DH || EPI == EPI_DHQ>(patch, patch_alt, acc, fetch, compute, store);
}

template <int EPI, int ACT, bool LUT = false, int NW = 4, typename Acc>
__device__ __forceinline__ void rows_epilogue(float* lds, float* lds_alt, const Acc& acc, const bf16_t* __restrict__ bias,
                                              int NC, int row0, int rows_valid, int e, int n0,
                                              const bf16_t* __restrict__ hpre_in, bf16_t* __restrict__ out0,
                                              bf16_t* __restrict__ out1, const lds_byte_t* lut = nullptr,
                                              const lds_int_t* smap = nullptr) {
  // the common case -- a whole tile, stored in place -- runs without store predicates
  const int wn = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6) & 1;
  const bool full = rows_valid == BM && NC - n0 - wn * (NB * 32) >= NB * 32;
#define FLEXMOE_EPI_CALL(BIAS, FULL, SCATTER) \
  rows_epilogue_t<EPI, ACT, LUT, BIAS, FULL, SCATTER, NW>(lds, lds_alt, acc, bias, NC, row0, rows_valid, e, n0, hpre_in, out0, out1, lut, smap)
  if (EPI == EPI_PLAIN && smap) {
    if (bias) FLEXMOE_EPI_CALL(true, false, true);
    else FLEXMOE_EPI_CALL(false, false, true);
  } else if (full) {
    if (bias) FLEXMOE_EPI_CALL(true, true, false);
    else FLEXMOE_EPI_CALL(false, true, false);
  } else {
    if (bias) FLEXMOE_EPI_CALL(true, false, false);
    else FLEXMOE_EPI_CALL(false, false, false);
  }
#undef FLEXMOE_EPI_CALL
}

// One output tile of rows_gemm: main loop and epilogue.  FULL = all eight 32-row blocks hold rows.
// (Kept as two separate instantiations with their own accumulators: merging the accumulators of
// a full-tile and a ragged-tile path costs hundreds of register copies.)
template <bool WT, int EPI, int ACT, bool FULL>
__device__ __forceinline__ void rows_tile(bf16_t* smem, const bf16_t* __restrict__ in, const bf16_t* __restrict__ w,
                                          const bf16_t* __restrict__ bias, int K, int NC, int row0, int rows_valid,
                                          int e, int n0, int cols_valid, const bf16_t* __restrict__ hpre_in,
                                          bf16_t* __restrict__ out0, bf16_t* __restrict__ out1) {
  const int nblk_rows = (rows_valid + 31) >> 5;
  const bf16_t* a_base = in + (size_t)row0 * K;
  const bf16_t* w_e = w + (size_t)e * K * NC;
  const int wave = threadIdx.x >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  f32x16 acc[MB][NB];
  zero_acc(acc);
  rows_mainloop<WT, FULL>(smem, acc, a_base, w_e, K, NC, n0, rows_valid, cols_valid, wm, wn, nblk_rows);

  rows_epilogue<EPI, ACT>((float*)smem, (float*)smem + kGemmThreads / kWave * (32 * 64), acc, bias, NC, row0, rows_valid, e, n0, hpre_in, out0, out1);
}

// flat row-tile index -> (vExpert, tile inside it): one wave scans the buckets' tile counts.
// Returns false (for the whole workgroup) when the workgroup has no tile.
struct RowTile {
  int row0, rows_valid, e, n0, cols_valid;
  int seg, nseg, slot;        // K segment of a split tile (nseg > 1) and its partial-tile slot
};
// Splitting the last, partly filled round of workgroups along K (plain-epilogue products with a long
// contraction).  With T valid tiles on 256 compute units, the tiles of the row tiles from
// r_split = floor(floor(T / 256) * 256 / col_tiles) on are the ones left for that last round; when
// they fill at most a quarter of the chip, each is contracted by S = 4 workgroups (K segments of equal
// length, a whole number of pipeline rounds each; S = 2 when they fill up to half of it): segment 0 by the tile's own workgroup, segments
// 1..S-1 by extra workgroups appended to the grid (block >= normal_grid).  Every segment leaves an
// fp32 partial tile; rows_split_reduce_kernel adds them in segment order (fixed order: results do
// not depend on scheduling).  The plan is a function of the bucket sizes: every workgroup derives
// the same one.
constexpr int kSplitMax = 4;
constexpr int kSplitUnits = 256;                      // compute units a round of workgroups fills
constexpr int kSplitMaxSlots = kSplitUnits;           // tail tiles x S <= 256
// In how many K segments the tail tiles are contracted: four when they then still fit one round of workgroups, else
// two, else one (no splitting); a segment is a whole number of pipeline rounds (four K tiles).
__host__ __device__ inline int split_factor(int full_rounds, int tail_tiles, int k_tiles) {
  if (full_rounds < 1 || tail_tiles <= 0) return 1;
  if (4 * tail_tiles <= kSplitUnits && k_tiles % 16 == 0) return 4;
  if (2 * tail_tiles <= kSplitUnits && k_tiles % 8 == 0) return 2;
  return 1;
}
struct SplitArg {
  unsigned normal_grid;      // blocks of the unsplit grid; 0 = no splitting
  int k_tiles;               // K / 32
  int tail_tile;             // >= 0: look up this tail tile (reduce kernel) instead of `block`
};
template <bool SPLIT = false>
__device__ __forceinline__ bool lookup_row_tile(const int32_t* __restrict__ voff, const int32_t* __restrict__ owner,
                                                int V, int NC, int row_tiles_max, int col_tiles, unsigned block,
                                                int* s_tile, RowTile* out, SplitArg sp = SplitArg{0, 0, -1}) {
  if (threadIdx.x < kWave) {
    const int lane = threadIdx.x;
    if (lane == 0) s_tile[0] = -1;
    const int per = (V + kWave - 1) / kWave;     // <= 8 buckets per lane
    int cnt[FLEXMOE_MAX_VEXPERTS / kWave], lo[FLEXMOE_MAX_VEXPERTS / kWave], hi[FLEXMOE_MAX_VEXPERTS / kWave];
    int own[FLEXMOE_MAX_VEXPERTS / kWave];
    int sum = 0;
#pragma unroll
    for (int q = 0; q < FLEXMOE_MAX_VEXPERTS / kWave; ++q) {
      const int v = lane * per + q;
      cnt[q] = lo[q] = hi[q] = own[q] = 0;
      if (q < per && v < V) {
        lo[q] = voff[v];
        hi[q] = voff[v + 1];
        own[q] = owner[v];                         // fetched now: no second round trip once the bucket is known
        cnt[q] = (hi[q] - lo[q] + BM - 1) / BM;
      }
      sum += cnt[q];
    }
    int incl = sum;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
      const int up = __shfl_up(incl, o);
      if (lane >= o) incl += up;
    }
    int rt = -1, ct = 0;
    int seg = 0, nseg = 1, slot = 0;
    if (SPLIT && sp.normal_grid) {
      const int rows_act = __shfl(incl, kWave - 1);
      const int full = rows_act * col_tiles / kSplitUnits;
      const int r_split = full * kSplitUnits / col_tiles;
      const int tail_tiles = (rows_act - r_split) * col_tiles;
      // (cutting in two pays since the kernels are persistent: -3.6 % on the GPT-medium-like step, whose second
      // forward product has 2.3 rounds of tiles; with one workgroup per tile it had measured no gain)
      const int S = split_factor(full, tail_tiles, sp.k_tiles);
      if (sp.tail_tile < 0 && block < sp.normal_grid) {
        if (!patched_tile(block, row_tiles_max, col_tiles, &rt, &ct)) rt = -1;
        if (S > 1 && rt >= r_split && rt < rows_act) {
          nseg = S;
          slot = ((rt - r_split) * col_tiles + ct) * S;
        }
      } else if (S > 1) {
        const int x = sp.tail_tile >= 0 ? sp.tail_tile * (S - 1) : (int)(block - sp.normal_grid);
        const int tt = x / (S - 1);
        if (tt < tail_tiles) {
          rt = r_split + tt / col_tiles;
          ct = tt % col_tiles;
          nseg = S;
          seg = 1 + x % (S - 1);
          slot = tt * S + seg;
        }
      }
    } else {
      if (!patched_tile(block, row_tiles_max, col_tiles, &rt, &ct)) rt = -1;
    }
    int start = incl - sum;
#pragma unroll
    for (int q = 0; q < FLEXMOE_MAX_VEXPERTS / kWave; ++q) {
      if (rt >= start && rt < start + cnt[q]) {
        const int row0 = lo[q] + (rt - start) * BM;
        s_tile[0] = row0;
        s_tile[1] = min(BM, hi[q] - row0);
        s_tile[2] = own[q];
        s_tile[3] = ct;
        if (SPLIT) {
          s_tile[4] = seg;
          s_tile[5] = nseg;
          s_tile[6] = slot;
        }
      }
      start += cnt[q];
    }
  }
  __syncthreads();
  if (s_tile[0] < 0) return false;                    // beyond the last tile (uniform)
  // workgroup-uniform values: keep them in scalar registers (scalar base addresses, scalar compares)
  out->row0 = __builtin_amdgcn_readfirstlane(s_tile[0]);
  out->rows_valid = __builtin_amdgcn_readfirstlane(s_tile[1]);
  out->e = __builtin_amdgcn_readfirstlane(s_tile[2]);
  out->n0 = __builtin_amdgcn_readfirstlane(s_tile[3] * BN);
  out->cols_valid = min(BN, NC - out->n0);
  out->seg = SPLIT ? __builtin_amdgcn_readfirstlane(s_tile[4]) : 0;
  out->nseg = SPLIT ? __builtin_amdgcn_readfirstlane(s_tile[5]) : 1;
  out->slot = SPLIT ? __builtin_amdgcn_readfirstlane(s_tile[6]) : 0;
  return true;
}

template <bool WT, int EPI, int ACT>
__global__ __launch_bounds__(kGemmThreads) void rows_gemm_bf16(
    const bf16_t* __restrict__ in, const bf16_t* __restrict__ w, const bf16_t* __restrict__ bias,
    const int32_t* __restrict__ voff, const int32_t* __restrict__ owner, int V, int K, int NC, int row_tiles_max,
    int col_tiles, const bf16_t* __restrict__ hpre_in, bf16_t* __restrict__ out0, bf16_t* __restrict__ out1) {
  __shared__ __align__(16) unsigned char smem_raw[kGemmLds];     // 128 KB of the 160 KB a compute unit has
  bf16_t* smem = (bf16_t*)smem_raw;
  __shared__ int s_tile[4];
  RowTile t;
  if (!lookup_row_tile(voff, owner, V, NC, row_tiles_max, col_tiles, blockIdx.x, s_tile, &t)) return;
  // Ragged tiles run the full-tile code (rows past the bucket are clamped on load and dropped
  // on store): skipping their empty 32-row MFMA blocks needs conditional MFMA groups, which the
  // register allocator only handles by spilling the accumulators.
  rows_tile<WT, EPI, ACT, true>(smem, in, w, bias, K, NC, t.row0, t.rows_valid, t.e, t.n0, t.cols_valid, hpre_in,
                                out0, out1);
}

}  // namespace flexmoe
