// bf16 expert FFN (paper Eq. 2) per vExpert bucket, forward and backward, as grouped GEMMs on
// the CDNA4 matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulation).
//
// All kernels share one 256x256 workgroup tile: 4 wavefronts (2x2), each owning a 128x128
// accumulator block = 16 MFMA tiles = 256 accumulator registers, one workgroup per compute unit.
//
//  * rows GEMMs: C[rows of bucket v, :] = In[rows of v, :] . W_owner(v)    (fwd GEMM1/GEMM2,
//    bwd dH and dXp).  The row dimension is cut per bucket: a device-side lookup maps the flat
//    row-tile index to (vExpert, tile inside it), so highly skewed bucket sizes need no host
//    synchronisation.  Rows of a ragged last tile are clamped on load and dropped on store.
//  * weight-gradient GEMMs: dW_e = sum over the vExperts v of e of L_v^T . R_v -- the contraction
//    runs over the tokens of every bucket of e in ascending vExpert id inside one accumulator,
//    which is the single-GPU image of the paper's replica gradient synchronisation.  Output tiles
//    are issued hottest expert first so the long contractions start early; when one expert's
//    contraction is much longer than the chip-wide average per compute unit it is cut into
//    segments that accumulate into fp32 partial tiles, summed in a fixed order by a second kernel
//    (the result does not depend on scheduling).
//
// Two operand pipelines:
//  * direct-to-LDS (rows_gemm_dma_bf16, wgrad_gemm_dma_bf16; used whenever K is a multiple of
//    128, i.e. for every benchmark shape): global_load_lds_dwordx4 copies 32-wide K tiles
//    straight into one of four LDS stages (no register staging, no LDS store instructions); an
//    operand whose contraction index is strided in memory is copied as stored and transposed on
//    the way out of LDS by ds_read_tr16_b64.  The loads of the tile three steps ahead are
//    spread between the MFMAs of the current one, and one LDS-only barrier per K tile orders
//    stage reuse.  The kernels are bound by L2 -> LDS bandwidth.
//  * register-staged (rows_gemm_bf16; any K that is a multiple of 8): 64-wide K
//    tiles through registers into two LDS stages, strided operands transposed 8x8 in registers.
//
// LDS tiles are XOR-swizzled at 16-byte chunk granularity so that fragment reads and tile
// writes are free of bank conflicts (measured: SQ_LDS_BANK_CONFLICT = 0).
// The MFMA is issued as (weights-fragment, activations-fragment) so that a lane ends up with 4
// consecutive output columns of one output row; the epilogue passes the accumulators through a
// wave-private LDS patch so that global stores fill whole 128-byte lines.
// GELU and its derivative act on bf16-rounded arguments, so both are read from a table indexed
// by the argument's bits (filled once per device from the fp64 formulas; outside the table's
// range GELU equals ReLU to below bf16 resolution).
#include <algorithm>
#include <mutex>

#include "common.h"

namespace flexmoe {

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int kGemmThreads = 256;
constexpr int MB = 4, NB = 4;                       // 32x32 MFMA tiles per wave: 4 x 4
constexpr int kTileElems = BM * BK;                 // one operand tile in LDS (elements)
constexpr size_t kGemmLds = 2 * 2 * kTileElems * sizeof(bf16_t);   // 2 stages x (A + B) = 128 KB

enum { EPI_FWD1 = 0, EPI_PLAIN = 1, EPI_DH = 2 };
#ifndef FLEXMOE_DMA_CPOL
#define FLEXMOE_DMA_CPOL ""      // cache-policy modifiers of the direct-to-LDS loads
#endif

union Frag8 {
  uint4 u;
  bf16x8 v;
};

__device__ __forceinline__ int swz(int row) { return (row ^ (row >> 3)) & 7; }
__device__ __forceinline__ int lds_off(int row, int chunk) { return row * BK + ((chunk ^ swz(row)) << 3); }

// ---- workgroup id -> tile, XCD aware ---------------------------------------------------------
// Workgroups are dealt round-robin to the 8 XCDs (id % 8), each with its own L2, and an XCD runs
// its workgroups in ascending id.  The rows x cols tile grid is cut into patches of ph x pw tiles
// (about 32 = one per CU of an XCD; pw divides cols whenever a divisor in 5..8 exists, so patches
// are full and every XCD gets the same work); the j-th workgroup of XCD x gets tile j % (ph*pw) of
// patch (j / (ph*pw)) * 8 + x.  The workgroups that run together on one XCD then share ph row
// operands and pw column operands in its L2, and the 8 patches in flight on the 8 XCDs are
// neighbours in the grid, so what they share is fetched from HBM once.
constexpr int kXcds = 8, kPatch = 32;
__host__ __device__ inline int patch_width(int cols) {
  if (cols <= 8) return cols;
  for (int pw = 8; pw >= 5; --pw)
    if (cols % pw == 0) return pw;
  return 8;
}
__host__ __device__ inline unsigned patched_grid(int rows, int cols) {
  const int pw = patch_width(cols), ph = kPatch / pw;
  const int np = ((rows + ph - 1) / ph) * ((cols + pw - 1) / pw);
  return (unsigned)((np + kXcds - 1) / kXcds * kXcds) * (ph * pw);
}
// returns false when the workgroup falls into the padding of the patch grid
__device__ __forceinline__ bool patched_tile(unsigned b, int rows, int cols, int* r, int* c) {
  const int pw = patch_width(cols), ph = kPatch / pw, psize = ph * pw;
  const int npc = (cols + pw - 1) / pw;
  const unsigned x = b % kXcds, j = b / kXcds;
  const unsigned P = (j / psize) * kXcds + x, q = j % psize;
  *r = (int)(P / npc) * ph + (int)(q / pw);
  *c = (int)(P % npc) * pw + (int)(q % pw);
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
// costs an absolute error below 2^-25.  Entries are computed in double precision on the device,
// once per device, and held as {r, q} fp32 pairs: 3457 entries, padded to 28 KB so that the GEMM
// kernels can pull the table into LDS with whole 1 KB direct loads.
constexpr int kLutLo = 103 << 7;                    // bf16 bits of 2^-24
constexpr int kLutHi = 130 << 7;                    // bf16 bits of 8.0
constexpr int kLutBytes = 28 * 1024;
constexpr int kLutEntries = kLutBytes / 8;
static_assert(kLutHi - kLutLo + 1 <= kLutEntries, "table does not fit its padding");
__device__ __align__(1024) float2 g_act_lut[2][kLutEntries];    // [0] erf form, [1] tanh form

__global__ void act_lut_init_kernel() {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= kLutEntries) return;
  const int m = min(kLutLo + i, kLutHi);
  const double a = (double)__uint_as_float((uint32_t)m << 16);
  double Fneg, dF;                                   // F(-a) and F'(a)
  if (blockIdx.y == 0) {
    Fneg = 0.5 * erfc(a * 0.70710678118654752440);
    dF = 0.39894228040143267794 * exp(-0.5 * a * a);
  } else {
    const double c = 0.79788456080286535588, u = c * (a + 0.044715 * a * a * a);
    const double th = tanh(u);
    Fneg = 0.5 * (1.0 - th);
    dF = 0.5 * (1.0 - th * th) * c * (1.0 + 3.0 * 0.044715 * a * a);
  }
  // r = -a F(-a);  GELU'(a) = F(a) + a F'(a) = 1 - F(-a) + a F'(a)
  g_act_lut[blockIdx.y][i] = make_float2((float)(-a * Fneg), (float)(a * dF - Fneg));
}

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
template <int EPI, int ACT> constexpr bool epilogue_uses_lut() { return EPI != EPI_PLAIN && ACT != FLEXMOE_RELU; }

// ---- epilogue ---------------------------------------------------------------------------------
// A lane's accumulators hold 4-column pieces of 32 different rows, which would make every global
// store touch 32 cache lines.  Instead the wave's 128x128 fp32 block goes out in eight rounds of
// 32 rows x 64 columns: accumulator registers -> one of two wave-private 8 KB LDS patches (16-byte chunks,
// chunk index XORed with row & 15: conflict free both ways) -> read back so that 16 lanes cover
// 64 consecutive columns of one row -> per-element epilogue in fp32 -> bf16 -> 8-byte stores that
// fill whole 128-byte lines.  The K loop ends with a barrier, so the LDS tiles are free.
// Per round, all eight 4-element pieces are first computed (compute(row in the wave's block
// (0..127), column in the wave's block (multiple of 4), float4 accumulators, uint2 side input)
// -> EpiOut, unconditional: straight-line code the scheduler can interleave) and then stored
// (store(row, col, EpiOut), where the ragged-edge predicates live).
// fetch(row, col) -> uint2: an optional per-element side input (the saved pre-activations of the
// backward epilogue); the fetches of round n+1 are issued before round n is processed so that
// their latency hides behind it.
struct EpiOut {
  uint2 a, b;
};
template <bool FETCH, typename Fetch, typename Compute, typename Store>
__device__ __forceinline__ void epilogue_rounds(float* patch0, float* patch1, const f32x16 (&acc)[MB][NB], Fetch fetch,
                                                Compute compute, Store store) {
  const int lane = threadIdx.x & 63;
  const int r = lane & 31, h = lane >> 5;
  const int rsub = lane >> 4, c = lane & 15;
  constexpr int kRounds = MB * (NB / 2);
  uint2 side[2][8];
  if (FETCH) {
#pragma unroll
    for (int it = 0; it < 8; ++it) side[0][it] = fetch(it * 4 + rsub, c * 4);
  }
  // Two patches per wave: round n+1's accumulators are written while round n is processed.  A
  // wave's LDS instructions execute in issue order, so the reads that follow the writes need no
  // wait, only a compiler barrier (the dependence runs across lanes, which the compiler cannot see).
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
  for (int i = 0; i < MB; ++i) {
#pragma unroll
    for (int jh = 0; jh < NB / 2; ++jh) {
      const int round = i * (NB / 2) + jh;
      float* patch = (round & 1) ? patch1 : patch0;
      if (FETCH && round + 1 < kRounds) {
        const int ni = (round + 1) / (NB / 2), njh = (round + 1) % (NB / 2);
#pragma unroll
        for (int it = 0; it < 8; ++it) side[(round + 1) & 1][it] = fetch(ni * 32 + it * 4 + rsub, njh * 64 + c * 4);
      }
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
        o[it] = compute(i * 32 + it * 4 + rsub, jh * 64 + c * 4, v[it], FETCH ? side[round & 1][it] : make_uint2(0, 0));
#pragma unroll
      for (int it = 0; it < 8; ++it) store(i * 32 + it * 4 + rsub, jh * 64 + c * 4, o[it]);
    }
  }
}

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
template <int EPI, int ACT, bool LUT, bool BIAS>
__device__ __forceinline__ void rows_epilogue_t(float* lds, float* lds_alt, const f32x16 (&acc)[MB][NB], const bf16_t* __restrict__ bias,
                                                int NC, int row0, int rows_valid, int e, int n0,
                                                const bf16_t* __restrict__ hpre_in, bf16_t* __restrict__ out0,
                                                bf16_t* __restrict__ out1, const lds_byte_t* lut,
                                                const lds_int_t* smap) {
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  float* patch = lds + wave * (32 * 64);
  float* patch_alt = lds_alt + wave * (32 * 64);
  const int col_base = n0 + wn * (NB * 32);
  // tile-relative 32-bit offsets on top of uniform per-tile base pointers (scalar base + vector
  // offset addressing instead of 64-bit vector address arithmetic per store)
  const size_t tile_base = (size_t)row0 * NC + col_base;
  const bf16_t* hpre_t = hpre_in + tile_base;
  bf16_t* out0_t = out0 + tile_base;
  bf16_t* out1_t = out1 + tile_base;
  const bf16_t* bias_t = bias + (size_t)e * NC + col_base;
  const int cols_left = NC - col_base;
  auto tile_row = [&](int row_w) { return (wm + 2 * (row_w >> 5)) * 32 + (row_w & 31); };
  auto fetch = [&](int row_w, int col_w) -> uint2 {
    const int lrow = tile_row(row_w);
    if (lrow < rows_valid && col_w < cols_left) return *(const uint2*)(hpre_t + (uint32_t)(lrow * NC + col_w));
    return make_uint2(0, 0);
  };
  auto compute = [&](int row_w, int col_w, float4 c, uint2 pre_in) -> EpiOut {
    EpiOut o;
    if (BIAS) {
      float b[4];
      unpack4(*(const uint2*)(bias_t + min(col_w, cols_left - 4)), b);
      c.x += b[0]; c.y += b[1]; c.z += b[2]; c.w += b[3];
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
  auto store = [&](int row_w, int col_w, const EpiOut& o) {
    const int lrow = tile_row(row_w);
    if (lrow < rows_valid && col_w < cols_left) {
      const uint32_t off = (uint32_t)(lrow * NC + col_w);
      if (EPI == EPI_PLAIN && smap) {
        // scattered store: tile row lrow is row smap[lrow] of the output (reverse routing of a top-1 layer)
        *(uint2*)(out0 + (size_t)smap[lrow] * NC + col_base + col_w) = o.a;
      } else if (EPI != EPI_FWD1 || out0) *(uint2*)(out0_t + off) = o.a;     // forward: the pre-activations are optional
      if (EPI != EPI_PLAIN) *(uint2*)(out1_t + off) = o.b;
    }
  };
  epilogue_rounds<EPI == EPI_DH>(patch, patch_alt, acc, fetch, compute, store);
}

template <int EPI, int ACT, bool LUT = false>
__device__ __forceinline__ void rows_epilogue(float* lds, float* lds_alt, const f32x16 (&acc)[MB][NB], const bf16_t* __restrict__ bias,
                                              int NC, int row0, int rows_valid, int e, int n0,
                                              const bf16_t* __restrict__ hpre_in, bf16_t* __restrict__ out0,
                                              bf16_t* __restrict__ out1, const lds_byte_t* lut = nullptr,
                                              const lds_int_t* smap = nullptr) {
  if (bias) rows_epilogue_t<EPI, ACT, LUT, true>(lds, lds_alt, acc, bias, NC, row0, rows_valid, e, n0, hpre_in, out0, out1, lut, smap);
  else rows_epilogue_t<EPI, ACT, LUT, false>(lds, lds_alt, acc, bias, NC, row0, rows_valid, e, n0, hpre_in, out0, out1, lut, smap);
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
// length, a whole number of pipeline rounds each): segment 0 by the tile's own workgroup, segments
// 1..S-1 by extra workgroups appended to the grid (block >= normal_grid).  Every segment leaves an
// fp32 partial tile; rows_split_reduce_kernel adds them in segment order (fixed order: results do
// not depend on scheduling).  The plan is a function of the bucket sizes: every workgroup derives
// the same one.
constexpr int kSplitMax = 4;
constexpr int kSplitUnits = 256;                      // compute units a round of workgroups fills
constexpr int kSplitMaxSlots = kSplitUnits;           // tail tiles x S <= 256
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
      // four segments or none: cutting in two (tails of 65 to 128 tiles) measured no faster than not
      // cutting, the fp32 round trip of the partial tiles eats what the shorter last round gains
      const int S = (full >= 1 && tail_tiles > 0 && kSplitMax * tail_tiles <= kSplitUnits &&
                     sp.k_tiles % (4 * kSplitMax) == 0) ? kSplitMax : 1;
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
  extern __shared__ __align__(16) unsigned char smem_raw[];
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

// =============================================================================================
// rows_gemm_dma: the same product for operands that are both contraction-contiguous
// (In [rows, K], W_e [NC, K]) and K a multiple of 128, with global -> LDS direct loads
// (global_load_lds, 16 bytes per lane, no register staging, no LDS store instructions).
// Four LDS stages of a 32-wide K tile (2 x 16 KB each): while tile t is multiplied, tiles
// t+1..t+3 are landed or in flight and tile t+4 is issued half-way through the step.  A direct load writes lane i's 16 bytes at
// the wave's LDS base + 16*i, so one instruction fills 16 rows x 64 bytes; the bank swizzle
// (16-byte chunk index XOR (row>>2)&3) is applied by choosing which global chunk a lane fetches.
// =============================================================================================
constexpr int DK = 32;
constexpr int kDmaStages = 4;
constexpr int kDmaTileBytes = 256 * DK * 2;            // one operand tile: 16 KB
constexpr int kDmaStageBytes = 2 * kDmaTileBytes;      // A + B

__device__ __forceinline__ int dma_off(int row, int c) { return row * (DK * 2) + ((c ^ ((row >> 2) & 3)) << 4); }

struct DmaSrc {
  const bf16_t* base;
  uint32_t off[4];
  __device__ __forceinline__ void init(const bf16_t* b, size_t ld, int rows_valid) {
    base = b;
    const int w = threadIdx.x >> 6, i = threadIdx.x & 63;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int row = (w * 4 + q) * 16 + (i >> 2);
      const int c = (i & 3) ^ ((row >> 2) & 3);
      off[q] = (uint32_t)(min(row, rows_valid - 1) * ld + c * 8);
    }
  }
  // The same tile with its rows gathered: tile row r is row rows[r] / k of the matrix at b (the
  // expert-wise layout transformation done on the fly: rows = the bucket's slice of `src`).
  __device__ __forceinline__ void init_gather(const bf16_t* b, size_t ld, const int32_t* __restrict__ rows, int k,
                                              int rows_valid) {
    base = b;
    const int w = threadIdx.x >> 6, i = threadIdx.x & 63;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int row = (w * 4 + q) * 16 + (i >> 2);
      const int c = (i & 3) ^ ((row >> 2) & 3);
      off[q] = (uint32_t)((size_t)(rows[min(row, rows_valid - 1)] / k) * ld + c * 8);
    }
  }
  // Fills the 16 KB LDS tile at `tile` with K columns k0..k0+31 of the operand's 256 rows.
  // The direct load is issued from inline assembly (M0 = LDS byte address of the wave's 1 KB
  // slice, lane i lands at M0 + 16*i): the compiler's wait-count insertion cannot tell which LDS
  // stage a direct load writes and would wait for every outstanding load before any LDS read;
  // here the waits are placed by hand (wait_vmcnt_le) before the barrier that publishes a stage.
  // q-th of the wave's four direct loads of one tile
  __device__ __forceinline__ void part(lds_byte_t* tile, int k0, int q) const {
    const unsigned w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const unsigned lds0 = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)tile) + w * 4096;
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
  uint32_t off[4];
  size_t ld;
  __device__ __forceinline__ void init(const bf16_t* b, size_t ld_, int cols_valid) {
    base = b;
    ld = ld_;
    const int w = threadIdx.x >> 6, i = threadIdx.x & 63;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int krow = (w * 4 + q) * 2 + (i >> 5);
      const int c = min(dmat_chunk(krow, i & 31), cols_valid / 8 - 1);
      off[q] = (uint32_t)(krow * ld + c * 8);
    }
  }
  __device__ __forceinline__ void part(lds_byte_t* tile, int k0, int q) const {
    const unsigned w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const unsigned lds0 = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)tile) + w * 4096;
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

// s_waitcnt vmcnt(8 * tiles) only (expcnt / lgkmcnt fields left at "no wait"): returns once at
// most `tiles` of the most recently issued K tiles (8 direct loads per wave each) are in flight.
__device__ __forceinline__ void wait_tiles_in_flight(int tiles) {
  if (tiles >= 3) __builtin_amdgcn_s_waitcnt(0x4F78);        // vmcnt(24)
  else if (tiles == 2) __builtin_amdgcn_s_waitcnt(0x4F70);   // vmcnt(16)
  else if (tiles == 1) __builtin_amdgcn_s_waitcnt(0x0F78);   // vmcnt(8)
  else __builtin_amdgcn_s_waitcnt(0x0F70);                   // vmcnt(0)
}

struct DmaFrags {
  Frag8 a[MB], b[NB];
};
// TRA / TRB: the operand's LDS tile is [k][256] (transposing reads) instead of [256][k].
template <bool TRA, bool TRB>
__device__ __forceinline__ void dma_read_frags(DmaFrags& f, const lds_byte_t* stage, int ks, int wm, int wn) {
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
  for (int j = 0; j < NB; ++j) {
    if (TRB) f.b[j].v = dmat_read_frag(Bs, (wn * NB + j) * 32, ks);
    else f.b[j].v = *(const __attribute__((address_space(3))) bf16x8*)(Bs + dma_off((wn * NB + j) * 32 + r, 2 * ks + h));
  }
}
__device__ __forceinline__ void dma_mma(f32x16 (&acc)[MB][NB], const DmaFrags& f) {
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j)
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.b[j].v, f.a[i].v, acc[i][j], 0, 0, 0);
}

// One K tile (two 16-wide k steps).  On entry f0 holds the fragments of (tile kt, k step 0).
// The barrier sits between the two k steps: before it the wave has fetched everything it needs
// from `cur`, so after it `cur` is free for tile kt+4; and tile kt+1 is published, so its first
// fragments can be fetched while the second k step's MFMAs run -- no LDS latency after the barrier.
// The direct loads are spread evenly between the MFMAs, one after every four (128 cycles of
// matrix-pipe work): the four waves share one address path, and a wave that issues its loads back
// to back leaves its matrix pipe idle while it queues there.  So a tile's eight loads per wave go
// out in two halves: loads 0..3 of tile kt+4 after the barrier of step kt (into `cur`, just
// freed), loads 4..7 before the barrier of step kt+1 (into that step's `prev`).
// Issue: begin() prepares the next tile in sequence, part(stage, q) starts its q-th direct load
// (q = 0..7) into `stage`, end() moves on to the tile after it.
// PRE: tile kt+3 exists (its second half is issued here).  POST: tile kt+4 exists.
// NEXT: tile kt+1 exists; WAIT = how many younger tiles may still be in flight once this wave's
// part of tile kt+1 has landed.
template <bool TRA, bool TRB, bool PRE, bool POST, int WAIT, bool NEXT, typename Issue>
__device__ __forceinline__ void dma_step(lds_byte_t* prev, lds_byte_t* cur, const lds_byte_t* nxt,
                                         f32x16 (&acc)[MB][NB], DmaFrags& f0, DmaFrags& f1, Issue& issue, int wm,
                                         int wn) {
  dma_read_frags<TRA, TRB>(f1, cur, 1, wm, wn);
#pragma unroll
  for (int i = 0; i < MB; ++i) {
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int j = 0; j < NB; ++j)
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f0.b[j].v, f0.a[i].v, acc[i][j], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    if (PRE) issue.part(prev, 4 + i);
  }
  if (PRE) issue.end();
  __builtin_amdgcn_sched_barrier(0);     // everything above is queued before the wave goes to wait
  if (NEXT) wait_tiles_in_flight(WAIT);
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
  if (NEXT) dma_read_frags<TRA, TRB>(f0, nxt, 0, wm, wn);
  if (POST) issue.begin();
#pragma unroll
  for (int i = 0; i < MB; ++i) {
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int j = 0; j < NB; ++j)
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f1.b[j].v, f1.a[i].v, acc[i][j], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    if (POST) issue.part(cur, i);
  }
}

// The whole K loop: KT tiles (a multiple of 4) through the four stages; the last four tiles,
// which have nothing left to prefetch, run as a peeled tail so that the steady-state loop body is
// branch-free.
template <bool TRA, bool TRB, typename Issue>
__device__ __forceinline__ void dma_pipeline(lds_byte_t* s0, lds_byte_t* s1, lds_byte_t* s2, lds_byte_t* s3,
                                             f32x16 (&acc)[MB][NB], Issue& issue, int KT, int wm, int wn) {
  lds_byte_t* const stages[4] = {s0, s1, s2, s3};
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    issue.begin();
#pragma unroll
    for (int q = 0; q < (t < 3 ? 8 : 4); ++q) issue.part(stages[t], q);   // tile 3: first half only
    if (t < 3) issue.end();
  }
  __builtin_amdgcn_s_waitcnt(0x4F74);                  // vmcnt(20): tile 0 has landed
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
  DmaFrags f0, f1;
  dma_read_frags<TRA, TRB>(f0, s0, 0, wm, wn);
  for (int kt = 0; kt < KT - 4; kt += 4) {
    dma_step<TRA, TRB, true, true, 2, true>(s3, s0, s1, acc, f0, f1, issue, wm, wn);
    dma_step<TRA, TRB, true, true, 2, true>(s0, s1, s2, acc, f0, f1, issue, wm, wn);
    dma_step<TRA, TRB, true, true, 2, true>(s1, s2, s3, acc, f0, f1, issue, wm, wn);
    dma_step<TRA, TRB, true, true, 2, true>(s2, s3, s0, acc, f0, f1, issue, wm, wn);
  }
  dma_step<TRA, TRB, true, false, 2, true>(s3, s0, s1, acc, f0, f1, issue, wm, wn);
  dma_step<TRA, TRB, false, false, 1, true>(s0, s1, s2, acc, f0, f1, issue, wm, wn);
  dma_step<TRA, TRB, false, false, 0, true>(s1, s2, s3, acc, f0, f1, issue, wm, wn);
  dma_step<TRA, TRB, false, false, 0, false>(s2, s3, s0, acc, f0, f1, issue, wm, wn);
  __syncthreads();                                     // all waves done with the last tile: LDS is free
}

// Tile sequence of the rows kernels: K tile t of both operands starts at contraction index 32 t.
template <typename WSrc> struct RowsIssue {
  const DmaSrc& a_src;
  const WSrc& w_src;
  int k_next;
  __device__ __forceinline__ void begin() {}
  __device__ __forceinline__ void part(lds_byte_t* stage, int q) const {
    if (q < 4) a_src.part(stage, k_next, q);
    else w_src.part(stage + kDmaTileBytes, k_next, q - 4);
  }
  __device__ __forceinline__ void end() { k_next += DK; }
};

template <bool WT, typename WSrc, int EPI, int ACT>
__device__ __forceinline__ void rows_dma_body(lds_byte_t* s0, lds_byte_t* s1, lds_byte_t* s2, lds_byte_t* s3,
                                              const RowTile& t, const bf16_t* __restrict__ in, const WSrc& w_src,
                                              const bf16_t* __restrict__ bias, int K, int NC,
                                              const bf16_t* __restrict__ hpre_in, bf16_t* __restrict__ out0,
                                              bf16_t* __restrict__ out1, const lds_byte_t* lut,
                                              const int32_t* __restrict__ gsrc, int gk,
                                              float* __restrict__ split_partial = nullptr,
                                              const int32_t* __restrict__ scatter_rows = nullptr) {
  const int wave = threadIdx.x >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  DmaSrc a_src;
  if (gsrc) a_src.init_gather(in, K, gsrc + t.row0, gk, t.rows_valid);
  else a_src.init(in + (size_t)t.row0 * K, K, t.rows_valid);
  f32x16 acc[MB][NB];
  zero_acc(acc);
  if (EPI == EPI_PLAIN && t.nseg > 1) {
    // one K segment of a split tile: fp32 partial tile (all 256 x 256 entries) for the reduce kernel
    const int kt = K / DK / t.nseg;
    RowsIssue<WSrc> issue{a_src, w_src, t.seg * kt * DK};
    dma_pipeline<false, !WT>(s0, s1, s2, s3, acc, issue, kt, wm, wn);
    float* out = split_partial + (size_t)t.slot * (BM * BN);
    float* patch = (float*)s0 + wave * (32 * 64);
    float* patch_alt = (float*)s1 + wave * (32 * 64);
    epilogue_rounds<false>(
        patch, patch_alt, acc, [](int, int) { return make_uint2(0, 0); },
        [](int, int, float4 c, uint2) {
          return EpiOut{make_uint2(__float_as_uint(c.x), __float_as_uint(c.y)),
                        make_uint2(__float_as_uint(c.z), __float_as_uint(c.w))};
        },
        [&](int row_w, int col_w, const EpiOut& o) {
          const int lrow = (wm + 2 * (row_w >> 5)) * 32 + (row_w & 31);
          *(uint4*)(out + lrow * BN + wn * (NB * 32) + col_w) = make_uint4(o.a.x, o.a.y, o.b.x, o.b.y);
        });
    return;
  }
  RowsIssue<WSrc> issue{a_src, w_src, 0};
  dma_pipeline<false, !WT>(s0, s1, s2, s3, acc, issue, K / DK, wm, wn);   // K % 128 == 0 (host check)
  const lds_int_t* smap = nullptr;
  if (EPI == EPI_PLAIN && scatter_rows) {
    // output rows of this tile (the epilogue's patches live in stages 0 and 1; stage 2 is free)
    lds_int_t* m = (lds_int_t*)s2;
    m[threadIdx.x] = scatter_rows[t.row0 + min((int)threadIdx.x, t.rows_valid - 1)];
    __syncthreads();
    smap = m;
  }
  rows_epilogue<EPI, ACT, epilogue_uses_lut<EPI, ACT>()>((float*)s0, (float*)s1, acc, bias, NC, t.row0, t.rows_valid, t.e, t.n0, hpre_in, out0,
                                                          out1, lut, smap);
}

// Arguments of one rows GEMM (device pointers; see rows_gemm_dma_bf16).
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

// One workgroup's tile of a rows GEMM; `block` is its index in that GEMM's (patched) grid.
template <bool WT, int EPI, int ACT>
__device__ __forceinline__ void rows_dma_block(const RowsDmaArgs& p, unsigned block, lds_byte_t* s0, lds_byte_t* s1,
                                               lds_byte_t* s2, lds_byte_t* s3, unsigned char* lut_lds, int* s_tile) {
  constexpr bool kLut = epilogue_uses_lut<EPI, ACT>();
  RowTile t;
  if (EPI == EPI_PLAIN) {
    const SplitArg sp{p.split_partial ? p.normal_grid : 0u, p.K / DK, -1};
    if (!lookup_row_tile<true>(p.voff, p.owner, p.V, p.NC, p.row_tiles_max, p.col_tiles, block, s_tile, &t, sp)) return;
  } else {
    if (!lookup_row_tile(p.voff, p.owner, p.V, p.NC, p.row_tiles_max, p.col_tiles, block, s_tile, &t)) return;
  }
  const lds_byte_t* lut = nullptr;
  if (kLut) {
    // the table rides in front of the operand tiles: its direct loads are the oldest in every
    // wave's queue, so the first wait of the K loop covers them and its barrier publishes them
    lut = (const lds_byte_t*)lut_lds;
    const unsigned w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const unsigned lds0 = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)lut) + w * (kLutBytes / 4);
    const unsigned char* g = (const unsigned char*)g_act_lut[ACT == FLEXMOE_GELU_ERF ? 0 : 1] + w * (kLutBytes / 4) +
                             (threadIdx.x & 63) * 16;
#pragma unroll
    for (int q = 0; q < kLutBytes / 4 / 1024; ++q) {
      const unsigned char* gq = g + q * 1024;
      asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" FLEXMOE_DMA_CPOL ::"v"(gq), "s"(lds0 + q * 1024) : "memory");
    }
  }
  const bf16_t* w_e = p.w + (size_t)t.e * p.K * p.NC;
  if (WT) {
    DmaSrc w_src;
    w_src.init(w_e + (size_t)t.n0 * p.K, p.K, t.cols_valid);
    rows_dma_body<true, DmaSrc, EPI, ACT>(s0, s1, s2, s3, t, p.in, w_src, p.bias, p.K, p.NC, p.hpre_in, p.out0, p.out1,
                                          lut, p.gsrc, p.gk, p.split_partial, p.scatter_rows);
  } else {
    DmaSrcT w_src;
    w_src.init(w_e + t.n0, p.NC, t.cols_valid);
    rows_dma_body<false, DmaSrcT, EPI, ACT>(s0, s1, s2, s3, t, p.in, w_src, p.bias, p.K, p.NC, p.hpre_in, p.out0,
                                            p.out1, lut, p.gsrc, p.gk, p.split_partial, p.scatter_rows);
  }
}

template <bool WT, int EPI, int ACT>
__global__ __launch_bounds__(kGemmThreads) void rows_gemm_dma_bf16(const RowsDmaArgs p) {
  __shared__ __align__(1024) unsigned char stage0[kDmaStageBytes];
  __shared__ __align__(1024) unsigned char stage1[kDmaStageBytes];
  __shared__ __align__(1024) unsigned char stage2[kDmaStageBytes];
  __shared__ __align__(1024) unsigned char stage3[kDmaStageBytes];
  __shared__ __align__(1024) unsigned char lut_lds[epilogue_uses_lut<EPI, ACT>() ? kLutBytes : 16];
  __shared__ int s_tile[8];
  rows_dma_block<WT, EPI, ACT>(p, blockIdx.x, (lds_byte_t*)stage0, (lds_byte_t*)stage1, (lds_byte_t*)stage2,
                               (lds_byte_t*)stage3, lut_lds, s_tile);
}

// Sum of the K segments of the split tail tiles (see lookup_row_tile): out = bf16(sum over
// segments in order + bias).  Grid: (kSplitSlices row slices of a tile, kSplitUnits / kSplitMax tail tiles).
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

// Work list of the weight-gradient kernels.  Experts are taken by descending load (ties by
// ascending id: the long contractions start first).  An expert's contraction runs over its
// non-empty buckets in ascending vExpert id, in K tiles of 32 tokens; with seg_tiles > 0 it is cut
// into segments of seg_tiles K tiles that different workgroups contract (a hot expert would
// otherwise be one long serial K loop): an expert with more than one segment leaves fp32 partial
// tiles in the workspace, `slot` numbering them, which wgrad_reduce_kernel adds up in segment
// order.  The whole list is a function of the bucket sizes only, so every workgroup re-derives it.
struct WgradJob {
  int e;        // expert, -1: no job
  int seg;      // segment of the expert's contraction
  int nseg;     // segments of this expert
  int slot;     // index of the expert's first partial tile set (meaningful when nseg > 1)
};
struct WgradShared {
  int cnt[FLEXMOE_MAX_VEXPERTS], own[FLEXMOE_MAX_VEXPERTS];
  int load[FLEXMOE_MAX_EXPERTS], tiles[FLEXMOE_MAX_EXPERTS];
  int rank_e[FLEXMOE_MAX_EXPERTS], rank_s[FLEXMOE_MAX_EXPERTS];
  int job[4];
  int nb;
  int bstart[FLEXMOE_MAX_VEXPERTS], brows[FLEXMOE_MAX_VEXPERTS];
};

// `want` counts segments in work-list order (rank-major).  Also fills sh.bstart/brows/nb with the
// expert's buckets.
// `table` (optional, [E] entries of {expert, segments, first slot, 0} by load rank) is written by the
// caller that passes it, for wgrad_reduce_kernel.
__device__ __forceinline__ WgradJob wgrad_plan(const int32_t* __restrict__ voff, const int32_t* __restrict__ owner,
                                               int E, int V, int seg_tiles, int want, WgradShared& sh,
                                               int4* __restrict__ table) {
  for (int v = threadIdx.x; v < V; v += kGemmThreads) {
    sh.cnt[v] = voff[v + 1] - voff[v];
    sh.own[v] = owner[v];
  }
  for (int e = threadIdx.x; e < E; e += kGemmThreads) {
    sh.load[e] = 0;
    sh.tiles[e] = 0;
  }
  if (threadIdx.x == 0) sh.job[0] = -1;
  __syncthreads();
  for (int v = threadIdx.x; v < V; v += kGemmThreads) {
    atomicAdd(&sh.load[sh.own[v]], sh.cnt[v]);
    atomicAdd(&sh.tiles[sh.own[v]], (sh.cnt[v] + DK - 1) / DK);
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
    // prefix over the ranks of the segment counts (and of the segment counts of split experts)
    const int lane = threadIdx.x;
    constexpr int kPer = FLEXMOE_MAX_EXPERTS / kWave;
    int sum = 0, sum_split = 0;
#pragma unroll
    for (int q = 0; q < kPer; ++q) {
      const int r = lane * kPer + q;
      const int n = r < E ? sh.rank_s[r] : 0;
      sum += n;
      sum_split += n > 1 ? n : 0;
    }
    int incl = sum, incl_split = sum_split;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
      const int up = __shfl_up(incl, o), up2 = __shfl_up(incl_split, o);
      if (lane >= o) {
        incl += up;
        incl_split += up2;
      }
    }
    int start = incl - sum, slot = incl_split - sum_split;
#pragma unroll
    for (int q = 0; q < kPer; ++q) {
      const int r = lane * kPer + q;
      const int n = r < E ? sh.rank_s[r] : 0;
      const bool hit = want >= start && want < start + n;
      if (hit) {
        sh.job[0] = sh.rank_e[r];
        sh.job[1] = want - start;
        sh.job[2] = n;
        sh.job[3] = slot;
      }
      if (table && r < E) table[r] = make_int4(sh.rank_e[r], n, slot, 0);
      start += n;
      slot += n > 1 ? n : 0;
    }
  }
  __syncthreads();
  WgradJob job{sh.job[0], sh.job[1], sh.job[2], sh.job[3]};
  if (job.e < 0) return job;                    // uniform
  if (threadIdx.x < kWave) {                   // the expert's non-empty buckets, ascending vExpert id
    const int lane = threadIdx.x;
    const unsigned long long lt = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    int nbw = 0;
    for (int vb = 0; vb < V; vb += kWave) {
      const int v = vb + lane;
      const bool hit = v < V && sh.own[v] == job.e && sh.cnt[v] > 0;
      const unsigned long long mask = __ballot(hit);
      if (hit) {
        const int pos = nbw + __popcll(mask & lt);
        sh.bstart[pos] = voff[v];
        sh.brows[pos] = sh.cnt[v];
      }
      nbw += __popcll(mask);
    }
    if (lane == 0) sh.nb = nbw;
  }
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
  uint32_t off[4];
  int krow[4];
  size_t ld;
  __device__ __forceinline__ void init(size_t ld_, int cols_valid) {
    ld = ld_;
    const int w = threadIdx.x >> 6, i = threadIdx.x & 63;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      krow[q] = (w * 4 + q) * 2 + (i >> 5);
      const int c = min(dmat_chunk(krow[q], i & 31), cols_valid / 8 - 1);
      off[q] = (uint32_t)(krow[q] * ld + c * 8);
    }
  }
  // `p`: token row 0 of this K tile, first column of the tile; rows >= k_valid come from kZeroRow
  __device__ __forceinline__ void part(lds_byte_t* tile, const bf16_t* __restrict__ p, int k_valid, int q) const {
    const unsigned w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const unsigned lds0 = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)tile) + w * 4096;
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
    if (q < 4) l_src.part(stage, lp, kv, q);
    else r_src.part(stage + kDmaTileBytes, rp, kv, q - 4);
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
  int4* table;
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
  const WgradJob job = wgrad_plan(p.voff, p.owner, p.E, p.V, seg_tiles, grow / m_tiles, sh, block == 0 ? p.table : nullptr);
  if (job.e < 0) return;
  const int nb = sh.nb;

  const int m0 = mt * BM, n0 = nt * BN;
  const int mvalid = min(BM, M - m0), nvalid = min(BN, NC - n0);
  const int wave = threadIdx.x >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  f32x16 acc[MB][NB];
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
    dma_pipeline<true, true>(s0, (lds_byte_t*)stage1, (lds_byte_t*)stage2, (lds_byte_t*)stage3, acc, issue, KT, wm, wn);
  }

  float* patch = (float*)stage0 + wave * (32 * 64);
  float* patch_alt = (float*)stage1 + wave * (32 * 64);
  const int col_base = n0 + wn * (NB * 32);
  auto tile_row = [&](int row_w) { return (wm + 2 * (row_w >> 5)) * 32 + (row_w & 31); };
  if (job.nseg == 1) {
    bf16_t* out = dw + (size_t)job.e * M * NC;
    epilogue_rounds<false>(
        patch, patch_alt, acc, [](int, int) { return make_uint2(0, 0); },
        [](int, int, float4 c, uint2) { return EpiOut{pack4(c.x, c.y, c.z, c.w), make_uint2(0, 0)}; },
        [&](int row_w, int col_w, const EpiOut& o) {
          const int lrow = tile_row(row_w);
          const int col = col_base + col_w;
          if (lrow < mvalid && col < NC) *(uint2*)(out + (size_t)(m0 + lrow) * NC + col) = o.a;
        });
  } else {
    // one of several segments: the fp32 tile goes to the workspace for wgrad_reduce_kernel
    float* out = partial + (size_t)(job.slot + job.seg) * M * NC;
    epilogue_rounds<false>(
        patch, patch_alt, acc, [](int, int) { return make_uint2(0, 0); },
        [](int, int, float4 c, uint2) {
          return EpiOut{make_uint2(__float_as_uint(c.x), __float_as_uint(c.y)),
                        make_uint2(__float_as_uint(c.z), __float_as_uint(c.w))};
        },
        [&](int row_w, int col_w, const EpiOut& o) {
          const int lrow = tile_row(row_w);
          const int col = col_base + col_w;
          if (lrow < mvalid && col < NC)
            *(uint4*)(out + (size_t)(m0 + lrow) * NC + col) = make_uint4(o.a.x, o.a.y, o.b.x, o.b.y);
        });
  }
}


__global__ __launch_bounds__(kGemmThreads) void wgrad_gemm_dma_bf16(const WgradDmaArgs p) {
  __shared__ __align__(1024) unsigned char stage0[kDmaStageBytes];
  __shared__ __align__(1024) unsigned char stage1[kDmaStageBytes];
  __shared__ __align__(1024) unsigned char stage2[kDmaStageBytes];
  __shared__ __align__(1024) unsigned char stage3[kDmaStageBytes];
  __shared__ WgradShared sh;
  wgrad_dma_block(p, blockIdx.x, stage0, stage1, stage2, stage3, sh);
}

// The three GEMMs of the backward pass that only depend on the dH kernel -- dXp = dHpre . W1^T,
// dW2 and dW1 -- as one launch: workgroups [0, n_dx) take dXp's tiles, the next n_w2 dW2's, the rest
// dW1's.  Each product alone ends in a partly filled last round of workgroups; in one grid the
// next product's tiles fill those compute units.  n_dx and n_w2 are multiples of 8, so every
// product keeps its workgroup -> XCD mapping.
__global__ __launch_bounds__(kGemmThreads) void bwd_tail_dma_bf16(const RowsDmaArgs dx, unsigned n_dx,
                                                                  const WgradDmaArgs g2, unsigned n_w2,
                                                                  const WgradDmaArgs g1) {
  __shared__ __align__(1024) unsigned char stage0[kDmaStageBytes];
  __shared__ __align__(1024) unsigned char stage1[kDmaStageBytes];
  __shared__ __align__(1024) unsigned char stage2[kDmaStageBytes];
  __shared__ __align__(1024) unsigned char stage3[kDmaStageBytes];
  __shared__ WgradShared sh;
  __shared__ int s_tile[8];
  const unsigned b = blockIdx.x;
  if (b < n_dx)
    rows_dma_block<true, EPI_PLAIN, FLEXMOE_RELU>(dx, b, (lds_byte_t*)stage0, (lds_byte_t*)stage1, (lds_byte_t*)stage2,
                                                   (lds_byte_t*)stage3, nullptr, s_tile);
  else
    wgrad_dma_block(b < n_dx + n_w2 ? g2 : g1, b < n_dx + n_w2 ? b - n_dx : b - n_dx - n_w2, stage0, stage1, stage2,
                    stage3, sh);
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
    out[i] = pack4(s4.x, s4.y, s4.z, s4.w);
  }
}

// =============================================================================================
// host side
// =============================================================================================
// Weight gradient: how many 32-token K tiles one workgroup contracts before the expert's sum is
// cut into a further segment: a compute unit's even share of all (output tile, K tile) pairs
// (shorter segments measured slower: more fp32 partial tiles), so that the hottest expert's contraction is no longer one serial K loop.  0 = no cutting:
// when a segment would hold more than a quarter of all tokens (many output tiles per expert: the
// grid is busy anyway, and the fp32 partial tiles would be large).
constexpr int kComputeUnits = 256;
static int wgrad_seg_tiles(int A, int d, int f) {
  const long long out_tiles = (long long)((d + BM - 1) / BM) * ((f + BN - 1) / BN);
  const long long k_tiles = A / DK;
  long long seg = k_tiles * out_tiles / kComputeUnits;
  if (seg < 32) seg = 32;
  return 4 * seg <= k_tiles ? (int)seg : 0;
}
// Upper bounds over all load distributions: extra segments (beyond one per expert), and partial
// tile sets (segments of experts that have more than one).
static int wgrad_extra_segments(int A, int V, int seg_tiles) { return seg_tiles ? (A / DK + V) / seg_tiles : 0; }
static int wgrad_partial_slots(int A, int V, int seg_tiles) { return seg_tiles ? 2 * ((A / DK + V) / seg_tiles) + 1 : 0; }
static size_t wgrad_table_bytes() { return FLEXMOE_MAX_EXPERTS * sizeof(int4); }

static int max_row_tiles(int A, int V) { return A / BM + V; }

// Partial tiles of the split last round (see lookup_row_tile): none for grids that can never fill a
// round of workgroups or whose contraction is short (the fp32 round trip would cost more than the idle
// compute units).
constexpr int kSplitMinK = 1024;
static size_t rows_split_bytes(int A, int V, int K, int NC) {
  if (K % 128 || K < kSplitMinK) return 0;
  if ((long long)max_row_tiles(A, V) * ((NC + BN - 1) / BN) <= kSplitUnits) return 0;
  return (size_t)kSplitMaxSlots * BM * BN * sizeof(float);
}

// Job table + fp32 partial tiles of one segmented weight-gradient product (0 when not segmented).
static size_t wgrad_tail_bytes(int A, int d, int f, int V) {
  const int seg_tiles = wgrad_seg_tiles(A, d, f);
  if (!seg_tiles) return 0;
  return align_up(wgrad_table_bytes() + (size_t)wgrad_partial_slots(A, V, seg_tiles) * d * f * sizeof(float), 256);
}

size_t ffn_ws_bytes(int A, int d, int f, int E, int V, int dtype) {
  const size_t s = dtype == FLEXMOE_BF16 ? 2 : 4;
  size_t need = align_up((size_t)A * f * s, 256) * 2;      // dHpre (or H in forward) + H
  if (dtype == FLEXMOE_BF16) {
    need += 2 * wgrad_tail_bytes(A, d, f, V);      // one region per weight gradient
    need += rows_split_bytes(A, V, f, d);          // GEMM2 / dXp: partial tiles of the split last round
  }
  return need;
}
static void* rows_split_ws(const FfnArgs& a, void* ws) {
  return (char*)ws + 2 * align_up((size_t)a.A * a.f * sizeof(bf16_t), 256) + 2 * wgrad_tail_bytes(a.A, a.d, a.f, a.V);
}

template <typename Kern> static hipError_t allow_big_lds(Kern kern) {
  return hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kGemmLds);
}


// Fills the activation tables of the current device the first time a kernel that reads them is
// launched there.  The fill runs on the caller's stream and is waited for before the device is
// marked ready (other streams may launch next); under stream capture nothing can be waited for,
// so the fill is recorded into the capture and the device stays unmarked.
static hipError_t ensure_act_lut(hipStream_t s) {
  static std::mutex mu;
  static bool ready[64] = {};
  int dev = 0;
  hipError_t err = hipGetDevice(&dev);
  if (err != hipSuccess) return err;
  std::lock_guard<std::mutex> lock(mu);
  if (dev < 64 && ready[dev]) return hipSuccess;
  hipLaunchKernelGGL(act_lut_init_kernel, dim3((kLutEntries + 255) / 256, 2), dim3(256), 0, s);
  err = hipGetLastError();
  if (err != hipSuccess) return err;
  hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
  err = hipStreamIsCapturing(s, &cap);
  if (err != hipSuccess) return err;
  if (cap != hipStreamCaptureStatusNone) return hipSuccess;
  err = hipStreamSynchronize(s);
  if (err == hipSuccess && dev < 64) ready[dev] = true;
  return err;
}

static RowsDmaArgs rows_dma_args(const FfnArgs& a, const void* in, const void* w, const void* bias, int K, int NC,
                                 const void* hpre_in, void* out0, void* out1, const int32_t* gsrc, int gk) {
  return RowsDmaArgs{(const bf16_t*)in, (const bf16_t*)w, (const bf16_t*)bias, a.voff, a.owner, a.V, K, NC,
                     max_row_tiles(a.A, a.V), (NC + BN - 1) / BN, (const bf16_t*)hpre_in, (bf16_t*)out0,
                     (bf16_t*)out1, gsrc, gk, nullptr, 0u, nullptr};
}

template <bool WT, int EPI, int ACT>
static hipError_t launch_rows_t(const FfnArgs& a, const void* in, const void* w, const void* bias, int K, int NC,
                                const void* hpre_in, void* out0, void* out1, hipStream_t s, const int32_t* gsrc, int gk,
                                void* split_ws, const int32_t* scatter_rows) {
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t err = allow_big_lds(rows_gemm_bf16<WT, EPI, ACT>);
    if (err != hipSuccess) return err;
    attr_done = true;
  }
  const int col_tiles = (NC + BN - 1) / BN;
  const int row_tiles = max_row_tiles(a.A, a.V);
  const unsigned grid = patched_grid(row_tiles, col_tiles);
  if (K % 128 == 0) {
    // K is a whole number of pipeline rounds: direct-to-LDS path
    if (epilogue_uses_lut<EPI, ACT>()) {
      hipError_t err = ensure_act_lut(s);
      if (err != hipSuccess) return err;
    }
    RowsDmaArgs p = rows_dma_args(a, in, w, bias, K, NC, hpre_in, out0, out1, gsrc, gk);
    p.scatter_rows = scatter_rows;
    if (EPI == EPI_PLAIN && split_ws && rows_split_bytes(a.A, a.V, K, NC)) {
      // the last, partly filled round of workgroups is cut along K: extra workgroups for the further
      // segments behind the normal grid, then the sum of the partial tiles
      p.split_partial = (float*)split_ws;
      p.normal_grid = grid;
      hipLaunchKernelGGL((rows_gemm_dma_bf16<WT, EPI, ACT>), dim3(grid + kSplitUnits), dim3(kGemmThreads), 0, s, p);
      hipLaunchKernelGGL(rows_split_reduce_kernel, dim3(kSplitSlices, kSplitUnits / kSplitMax), dim3(kGemmThreads), 0, s, p);
      return hipGetLastError();
    }
    hipLaunchKernelGGL((rows_gemm_dma_bf16<WT, EPI, ACT>), dim3(grid), dim3(kGemmThreads), 0, s, p);
    return hipGetLastError();
  }
  if (gsrc || scatter_rows) return hipErrorInvalidValue;   // gathered / scattered rows only on the direct-to-LDS path (host check upstream)
  hipLaunchKernelGGL((rows_gemm_bf16<WT, EPI, ACT>), dim3(grid), dim3(kGemmThreads), kGemmLds, s, (const bf16_t*)in,
                     (const bf16_t*)w, (const bf16_t*)bias, a.voff, a.owner, a.V, K, NC, row_tiles, col_tiles,
                     (const bf16_t*)hpre_in, (bf16_t*)out0, (bf16_t*)out1);
  return hipGetLastError();
}

template <bool WT, int EPI>
static hipError_t launch_rows(const FfnArgs& a, const void* in, const void* w, const void* bias, int K, int NC,
                              const void* hpre_in, void* out0, void* out1, hipStream_t s,
                              const int32_t* gsrc = nullptr, int gk = 1, void* split_ws = nullptr,
                              const int32_t* scatter_rows = nullptr) {
  if (EPI == EPI_PLAIN)
    return launch_rows_t<WT, EPI, FLEXMOE_RELU>(a, in, w, bias, K, NC, hpre_in, out0, out1, s, gsrc, gk, split_ws,
                                                scatter_rows);
  switch (a.act) {
    case FLEXMOE_RELU:
      return launch_rows_t<WT, EPI, FLEXMOE_RELU>(a, in, w, bias, K, NC, hpre_in, out0, out1, s, gsrc, gk, nullptr, nullptr);
    case FLEXMOE_GELU_ERF:
      return launch_rows_t<WT, EPI, FLEXMOE_GELU_ERF>(a, in, w, bias, K, NC, hpre_in, out0, out1, s, gsrc, gk, nullptr, nullptr);
    default:
      return launch_rows_t<WT, EPI, FLEXMOE_GELU_TANH>(a, in, w, bias, K, NC, hpre_in, out0, out1, s, gsrc, gk, nullptr, nullptr);
  }
}

// One weight-gradient product's arguments and grid; `ws_tail` holds its job table and fp32 partial
// tiles when the contraction is cut into segments (wgrad_tail_bytes each).
static WgradDmaArgs wgrad_dma_args(const FfnArgs& a, const void* L, const void* R, int M, int NC, void* dw,
                                   void* ws_tail, unsigned* grid) {
  const int m_tiles = (M + BM - 1) / BM, n_tiles = (NC + BN - 1) / BN;
  const int seg_tiles = wgrad_seg_tiles(a.A, a.d, a.f);
  int4* table = seg_tiles ? (int4*)ws_tail : nullptr;
  float* partial = seg_tiles ? (float*)((char*)ws_tail + wgrad_table_bytes()) : nullptr;
  const int seg_rows_max = a.E + wgrad_extra_segments(a.A, a.V, seg_tiles);
  *grid = patched_grid(seg_rows_max * m_tiles, n_tiles);
  return WgradDmaArgs{(const bf16_t*)L, (const bf16_t*)R, a.voff, a.owner, a.E, a.V, M, NC, m_tiles, n_tiles,
                      seg_tiles, seg_rows_max, partial, table, (bf16_t*)dw};
}

static void launch_wgrad_reduce(const FfnArgs& a, const WgradDmaArgs& g, hipStream_t s) {
  if (!g.seg_tiles) return;
  const int blocks = (int)std::min<size_t>(((size_t)g.M * g.NC / 4 + kGemmThreads - 1) / kGemmThreads, 2048);
  hipLaunchKernelGGL(wgrad_reduce_kernel, dim3(blocks, a.E), dim3(kGemmThreads), 0, s, (const int4*)g.table, g.M, g.NC,
                     (const float*)g.partial, g.dw);
}

static hipError_t launch_wgrad(const FfnArgs& a, const void* L, const void* R, int M, int NC, void* dw, void* ws_tail,
                               hipStream_t s) {
  unsigned grid;
  const WgradDmaArgs g = wgrad_dma_args(a, L, R, M, NC, dw, ws_tail, &grid);
  hipLaunchKernelGGL(wgrad_gemm_dma_bf16, dim3(grid), dim3(kGemmThreads), 0, s, g);
  launch_wgrad_reduce(a, g, s);
  return hipGetLastError();
}

hipError_t launch_ffn_fwd_bf16(const FfnArgs& a, const void* xp, const void* w1, const void* b1, const void* w2,
                               const void* b2, void* hpre, void* yp, void* ws, hipStream_t s) {
  if (a.A == 0) return hipSuccess;
  void* h = ws;
  hipError_t err = launch_rows<false, EPI_FWD1>(a, xp, w1, b1, a.d, a.f, nullptr, hpre, h, s);
  if (err != hipSuccess) return err;
  return launch_rows<false, EPI_PLAIN>(a, h, w2, b2, a.f, a.d, nullptr, yp, nullptr, s, nullptr, 1, rows_split_ws(a, ws));
}

// Forward with the expert-wise layout transformation folded into GEMM1's row loads: bucket row p
// is row src[p] / k of x.  d must be a multiple of 128 (direct-to-LDS path).
hipError_t launch_ffn_fwd_gather_bf16(const FfnArgs& a, const void* x, const int32_t* src, int k, const void* w1,
                                      const void* b1, const void* w2, const void* b2, void* hpre, void* yp, void* ws,
                                      hipStream_t s) {
  if (a.A == 0) return hipSuccess;
  void* h = ws;
  hipError_t err = launch_rows<false, EPI_FWD1>(a, x, w1, b1, a.d, a.f, nullptr, hpre, h, s, src, k);
  if (err != hipSuccess) return err;
  return launch_rows<false, EPI_PLAIN>(a, h, w2, b2, a.f, a.d, nullptr, yp, nullptr, s, nullptr, 1, rows_split_ws(a, ws));
}

// The expert path of a top-1 layer without Xp and Yp: rows gathered through src on load (as above)
// and the second product's rows stored straight to y[src[p], :] -- with one expert per token the gate
// weight is exactly 1, so this is flexmoe_combine folded into the epilogue.  d and f multiples of 128.
hipError_t launch_ffn_fwd_top1_bf16(const FfnArgs& a, const void* x, const int32_t* src, const void* w1, const void* b1,
                                    const void* w2, const void* b2, void* hpre, void* y, void* ws, hipStream_t s) {
  if (a.A == 0) return hipSuccess;
  void* h = ws;
  hipError_t err = launch_rows<false, EPI_FWD1>(a, x, w1, b1, a.d, a.f, nullptr, hpre, h, s, src, 1);
  if (err != hipSuccess) return err;
  return launch_rows<false, EPI_PLAIN>(a, h, w2, b2, a.f, a.d, nullptr, y, nullptr, s, nullptr, 1, rows_split_ws(a, ws), src);
}

hipError_t launch_ffn_bwd_bf16(const FfnArgs& a, const void* dyp, const void* xp, const void* hpre, const void* w1,
                               const void* w2, void* dxp, void* dw1, void* dw2, void* ws, hipStream_t s) {
  bf16_t* dhpre = (bf16_t*)ws;
  bf16_t* h = (bf16_t*)((char*)ws + align_up((size_t)a.A * a.f * sizeof(bf16_t), 256));
  hipError_t err;
  if (a.A > 0) {
    // dH = dYp . W2^T fused with act'(Hpre); W2_e is [f, d], contraction index d contiguous
    err = launch_rows<true, EPI_DH>(a, dyp, w2, nullptr, a.d, a.f, hpre, dhpre, h, s);
    if (err != hipSuccess) return err;
  }
  // dW2 = H^T . dYp, dW1 = Xp^T . dHpre: each with its own table and partial tiles
  void* ws_tail2 = (char*)ws + 2 * align_up((size_t)a.A * a.f * sizeof(bf16_t), 256);
  void* ws_tail1 = (char*)ws_tail2 + wgrad_tail_bytes(a.A, a.d, a.f, a.V);
  // dXp, dW2 and dW1 share one launch when dXp's contraction is a whole number of pipeline rounds and
  // its grid is only a few rounds of workgroups (the partly filled last round is then a visible
  // share of it; with many rounds keeping each product's tiles to themselves is faster: measured
  // -3 % on the backward pass at 1.2 rounds, -1 % at 2.4, +1.7 % at 17.5)
  const unsigned dx_tiles = patched_grid(max_row_tiles(a.A, a.V), (a.d + BN - 1) / BN);
  if (a.A > 0 && a.f % 128 == 0 && dx_tiles <= 8 * 256) {
    auto round8 = [](unsigned n) { return (n + 7u) & ~7u; };
    unsigned grid2, grid1;
    const RowsDmaArgs dx = rows_dma_args(a, dhpre, w1, nullptr, a.f, a.d, nullptr, dxp, nullptr, nullptr, 1);
    const WgradDmaArgs g2 = wgrad_dma_args(a, h, dyp, a.f, a.d, dw2, ws_tail2, &grid2);
    const WgradDmaArgs g1 = wgrad_dma_args(a, xp, dhpre, a.d, a.f, dw1, ws_tail1, &grid1);
    const unsigned n_dx = round8(patched_grid(dx.row_tiles_max, dx.col_tiles)), n_w2 = round8(grid2);
    hipLaunchKernelGGL(bwd_tail_dma_bf16, dim3(n_dx + n_w2 + grid1), dim3(kGemmThreads), 0, s, dx, n_dx, g2, n_w2, g1);
    launch_wgrad_reduce(a, g2, s);
    launch_wgrad_reduce(a, g1, s);
    return hipGetLastError();
  }
  if (a.A > 0) {
    // dXp = dHpre . W1^T; W1_e is [d, f], contraction index f contiguous
    err = launch_rows<true, EPI_PLAIN>(a, dhpre, w1, nullptr, a.f, a.d, nullptr, dxp, nullptr, s, nullptr, 1,
                                       rows_split_ws(a, ws));
    if (err != hipSuccess) return err;
  }
  err = launch_wgrad(a, h, dyp, a.f, a.d, dw2, ws_tail2, s);
  if (err != hipSuccess) return err;
  return launch_wgrad(a, xp, dhpre, a.d, a.f, dw1, ws_tail1, s);
}

}  // namespace flexmoe
