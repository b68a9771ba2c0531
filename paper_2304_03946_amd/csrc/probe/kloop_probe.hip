// Ceilings of the grouped-GEMM K loop on one MI355X (gfx950), measured with stripped copies of the loop: no tile
// lookup, no epilogue, no tile turnover, 256 workgroups of 4 waves (one per compute unit), each wave a 128 x 128
// accumulator block, operands through four 32 KB LDS stages fed by direct-to-LDS loads (global_load_lds_dwordx4),
// fragments double-buffered, the eight loads of a tile spread between the MFMAs, one LDS-only barrier per K tile.
// Every variant is run with constant operand bits (no toggling: the chip holds its clock, so stalls show) and with
// random mantissas and signs (the matrix pipes then run into the power limit).  Prints TFLOP/s per variant:
//   A  MFMA only, v_mfma_f32_32x32x16_bf16 against v_mfma_f32_16x16x32_bf16
//   B  the loop with contiguous 1 KB loads (whole 128-byte lines), S workgroups of an XCD walking the same stream
//      (the first one misses the XCD's L2, the others hit): S = 32, 16, 8, 4, 2
//   C  the loop with the access pattern of a row-major operand (row pitch 16 KB, 64 bytes of 16 rows per load: half
//      lines), 4 x 8 tiles per XCD sharing rows as the real kernels do; and the same bytes as whole lines
//   D  256 x 128 tiles, two workgroups per compute unit (three stages of 24 KB each), contiguous and row-major
//   E  the 256 x 256 tile on eight waves (two per SIMD, 128 x 64 accumulator blocks)
//   F  E with v_mfma_f32_16x16x32_bf16 and the fragment schedule the kernels use with it; and, to price the loop's
//      parts, the same loop without its barrier, without its direct loads (after the first three tiles: the stages keep
//      what they hold), without its LDS reads (fragments stay what they are), and without any of them.  These
//      variants compute nothing meaningful; every LDS and global address stays what it is in the full loop.
// Build: paper_2304_03946_amd/build.py builds it next to the library; run: paper_2304_03946_amd/kloop_probe
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) unsigned char lds_byte_t;
#define CHECK(x)                                                           \
  do {                                                                     \
    hipError_t e = (x);                                                    \
    if (e != hipSuccess) {                                                 \
      printf("error %s at line %d\n", hipGetErrorString(e), __LINE__);     \
      return 1;                                                            \
    }                                                                      \
  } while (0)
#define DMA(p, ldsaddr) asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(p), "s"(ldsaddr) : "memory")

__device__ __forceinline__ int dma_off(int row, int c) { return row * 64 + ((c ^ ((row >> 2) & 3)) << 4); }
// the swizzle that keeps the 16 x 16 x 32 instruction's fragment reads (row = lane % 16, chunk = lane / 16) free of bank conflicts
__device__ __forceinline__ int dma_off16(int row, int c) { return row * 64 + ((c ^ ((row >> 1) & 3)) << 4); }
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}
__device__ __forceinline__ uint32_t hash32(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
  return x;
}
// bf16 pairs: 0.125 (constant) or random sign and mantissa with that exponent (no NaN, no overflow in the sums)
__device__ __forceinline__ uint32_t operand_bits(uint32_t seed, int random) {
  return random ? ((hash32(seed) & 0x80ff80ffu) | 0x3e003e00u) : 0x3e003e00u;
}
__global__ void fill_kernel(uint32_t* g, size_t n, int random) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
    g[i] = operand_bits((uint32_t)i * 2654435761u, random);
}
union F8 {
  uint32_t u[4];
  bf16x8 v;
};

// ---- A: MFMA only ------------------------------------------------------------------------------------------
template <int SHAPE>
__global__ __launch_bounds__(256) void mfma_only(float* out, int iters, int random) {
  F8 a[8], b[8];
  for (int i = 0; i < 8; ++i)
    for (int q = 0; q < 4; ++q) {
      a[i].u[q] = operand_bits(threadIdx.x * 128 + i * 4 + q + blockIdx.x * 7919, random);
      b[i].u[q] = operand_bits(threadIdx.x * 128 + 64 + i * 4 + q + blockIdx.x * 104729, random);
    }
  float s = 0.f;
  if (SHAPE == 32) {
    f32x16 acc[4][4];
    for (int i = 0; i < 4; ++i) for (int j = 0; j < 4; ++j) for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.f;
    for (int it = 0; it < iters; ++it)
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[j].v, a[i].v, acc[i][j], 0, 0, 0);
    for (int i = 0; i < 4; ++i) for (int j = 0; j < 4; ++j) for (int q = 0; q < 16; ++q) s += acc[i][j][q];
  } else {
    f32x4 acc[8][8];
    for (int i = 0; i < 8; ++i) for (int j = 0; j < 8; ++j) for (int q = 0; q < 4; ++q) acc[i][j][q] = 0.f;
    for (int it = 0; it < iters; ++it)
#pragma unroll
      for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b[j].v, a[i].v, acc[i][j], 0, 0, 0);
    for (int i = 0; i < 8; ++i) for (int j = 0; j < 8; ++j) for (int q = 0; q < 4; ++q) s += acc[i][j][q];
  }
  if (s == 123.456f) out[threadIdx.x] = s;      // keeps the loop alive; never true
}

// ---- B, C, D: the K loop -----------------------------------------------------------------------------------
// NBW = 32-column blocks per wave (4: tile 256 x 256, 2: tile 256 x 128); STAGES = LDS stages.
// PATTERN 0: contiguous stream, `share` workgroups of an XCD on the same stream; 1: row-major operands with a 16 KB
// row pitch, 64 bytes of 16 rows per load; 2: the same bytes fetched as whole lines (128 bytes of 8 rows per load).
struct LoopArgs {
  float* out;
  const unsigned char* g;
  int iters, share;
  size_t window;
};
template <int NBW, int STAGES, int PATTERN>
__device__ __forceinline__ void loop_body(const LoopArgs p) {
  constexpr int kStage = 16384 + NBW * 4096;
  constexpr int kLoads = 4 + NBW;
  constexpr size_t kPitch = 16384;
  __shared__ __attribute__((aligned(1024))) unsigned char lds[STAGES * kStage];
  for (int i = threadIdx.x; i < STAGES * kStage / 4; i += 256) ((uint32_t*)lds)[i] = 0x3e003e00u;
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, wm = wave >> 1, wn = wave & 1;
  const int r = lane & 31, h = lane >> 5;
  const int x = blockIdx.x % 8, j = blockIdx.x / 8;
  // contiguous pattern: stream base and start offset inside the window
  const unsigned char* gp = p.g + ((size_t)x * (32 / p.share) + (j % 32) / p.share) * p.window + threadIdx.x * 16;
  size_t goff = ((size_t)(j % p.share) * 65536) % p.window;
  if (goff + kStage > p.window) goff = 0;
  // row-major pattern: the XCD works on 4 row tiles x (8 or 16) column tiles; 1024 + 2048 rows of 16 KB per XCD
  const int ct = NBW == 4 ? 8 : 16, jj = j % (4 * ct);
  const unsigned char* abase = p.g + ((size_t)x * 3072 + (jj / ct) * 256) * kPitch;
  const unsigned char* bbase = p.g + ((size_t)x * 3072 + 1024 + (jj % ct) * (64 * NBW)) * kPitch;
  size_t aoff[4], boff[NBW];
  for (int q = 0; q < 4; ++q) {
    const int row = PATTERN == 2 ? (wave * 4 + q) * 16 + (lane >> 3) * 2 : (wave * 4 + q) * 16 + (lane >> 2);
    aoff[q] = (size_t)row * kPitch + (PATTERN == 2 ? (lane & 7) * 16 : (lane & 3) * 16);
  }
  for (int q = 0; q < NBW; ++q) {
    const int row = PATTERN == 2 ? (wave * NBW + q) * 16 + (lane >> 3) * 2 : (wave * NBW + q) * 16 + (lane >> 2);
    boff[q] = (size_t)row * kPitch + (PATTERN == 2 ? (lane & 7) * 16 : (lane & 3) * 16);
  }
  f32x16 acc[4][NBW];
  for (int i = 0; i < 4; ++i) for (int c = 0; c < NBW; ++c) for (int q = 0; q < 16; ++q) acc[i][c][q] = 0.f;
  bf16x8 a0[4], b0[NBW], a1[4], b1[NBW];
  auto frags = [&](bf16x8 (&a)[4], bf16x8 (&b)[NBW], const lds_byte_t* st, int ks) {
#pragma unroll
    for (int i = 0; i < 4; ++i) a[i] = *(const __attribute__((address_space(3))) bf16x8*)(st + dma_off((wm + 2 * i) * 32 + r, 2 * ks + h));
#pragma unroll
    for (int c = 0; c < NBW; ++c) b[c] = *(const __attribute__((address_space(3))) bf16x8*)(st + 16384 + dma_off((wn * NBW + c) * 32 + r, 2 * ks + h));
  };
  const unsigned lds0 = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)(lds_byte_t*)lds);
  const unsigned wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  int ktile = 0;
  auto issue = [&](int stage, int q) {
    if (PATTERN == 0) {
      const unsigned char* src = gp + goff + q * 4096;
      DMA(src, lds0 + stage * kStage + q * 4096 + wv * 1024);
    } else {
      const size_t koff = PATTERN == 2 ? (size_t)(ktile & 127) * 128 : (size_t)(ktile & 255) * 64;
      if (q < 4) {
        const unsigned char* src = abase + aoff[q] + koff;
        DMA(src, lds0 + stage * kStage + wv * 4096 + q * 1024);
      } else {
        const unsigned char* src = bbase + boff[q - 4] + koff;
        DMA(src, lds0 + stage * kStage + 16384 + wv * (NBW * 1024) + (q - 4) * 1024);
      }
    }
  };
  auto advance = [&]() {
    goff += kStage;
    if (goff + kStage > p.window) goff = 0;      // the next tile must end inside the window
    ++ktile;
  };
  for (int t = 0; t < STAGES - 1; ++t) {
    for (int q = 0; q < kLoads; ++q) issue(t, q);
    advance();
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);
  lds_barrier();
  frags(a0, b0, (const lds_byte_t*)lds, 0);
  int cur = 0;
  for (int it = 0; it < p.iters; ++it) {
    const lds_byte_t* st = (const lds_byte_t*)lds + cur * kStage;
    const int nxt = cur + 1 == STAGES ? 0 : cur + 1;
    const int fill_stage = cur == 0 ? STAGES - 1 : cur - 1;      // consumed by the previous iteration
    frags(a1, b1, st, 1);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int c = 0; c < NBW; ++c) acc[i][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b0[c], a0[i], acc[i][c], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int q = i * kLoads / 4; q < (i + 1) * kLoads / 4; ++q) issue(fill_stage, q);
    }
    advance();
    __builtin_amdgcn_sched_barrier(0);
    if (STAGES == 4) __builtin_amdgcn_s_waitcnt(0x4F70);      // vmcnt(16): the next tile has landed, two younger in flight
    else __builtin_amdgcn_s_waitcnt(0x0F76);                  // vmcnt(6): one younger tile of six loads in flight
    lds_barrier();
    frags(a0, b0, (const lds_byte_t*)lds + nxt * kStage, 0);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int c = 0; c < NBW; ++c) acc[i][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b1[c], a1[i], acc[i][c], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    cur = nxt;
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);
  __syncthreads();
  float s = 0.f;
  for (int i = 0; i < 4; ++i) for (int c = 0; c < NBW; ++c) for (int q = 0; q < 16; ++q) s += acc[i][c][q];
  if (s == 123.456f) p.out[threadIdx.x] = s;
}
template <int PATTERN>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void loop_256x256(const LoopArgs p) { loop_body<4, 4, PATTERN>(p); }
template <int PATTERN>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void loop_256x128(const LoopArgs p) { loop_body<2, 3, PATTERN>(p); }

// ---- E: the same 256 x 256 tile and LDS stages with eight waves (two per SIMD) ----------------------------------
// Wave w covers rows (wm + 2 i) * 32, i < 4, and two 32-column blocks: 128 x 64 outputs = 128 accumulator registers,
// so two waves fit a SIMD and one can issue while the other waits.  Contiguous loads, four per wave and K tile.
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2))) void loop_256x256_8waves(const LoopArgs p) {
  constexpr int kStage = 32768, STAGES = 4;
  __shared__ __attribute__((aligned(1024))) unsigned char lds[STAGES * kStage];
  for (int i = threadIdx.x; i < STAGES * kStage / 4; i += 512) ((uint32_t*)lds)[i] = 0x3e003e00u;
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, wm = (wave >> 1) & 1, wn = wave & 1, hh = wave >> 2;
  const int r = lane & 31, h = lane >> 5;
  const int x = blockIdx.x % 8, j = blockIdx.x / 8;
  const unsigned char* gp = p.g + ((size_t)x * (32 / p.share) + (j % 32) / p.share) * p.window + threadIdx.x * 16;
  size_t goff = ((size_t)(j % p.share) * 65536) % p.window;
  if (goff + kStage > p.window) goff = 0;
  f32x16 acc[4][2];
  for (int i = 0; i < 4; ++i) for (int c = 0; c < 2; ++c) for (int q = 0; q < 16; ++q) acc[i][c][q] = 0.f;
  bf16x8 a0[4], b0[2], a1[4], b1[2];
  auto frags = [&](bf16x8 (&a)[4], bf16x8 (&b)[2], const lds_byte_t* st, int ks) {
#pragma unroll
    for (int i = 0; i < 4; ++i) a[i] = *(const __attribute__((address_space(3))) bf16x8*)(st + dma_off((wm + 2 * i) * 32 + r, 2 * ks + h));
#pragma unroll
    for (int c = 0; c < 2; ++c) b[c] = *(const __attribute__((address_space(3))) bf16x8*)(st + 16384 + dma_off((wn * 4 + hh * 2 + c) * 32 + r, 2 * ks + h));
  };
  const unsigned lds0 = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)(lds_byte_t*)lds);
  const unsigned wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  auto issue = [&](int stage, int q) {
    const unsigned char* src = gp + goff + q * 8192;
    DMA(src, lds0 + stage * kStage + q * 8192 + wv * 1024);
  };
  auto advance = [&]() {
    goff += kStage;
    if (goff + kStage > p.window) goff = 0;
  };
  for (int t = 0; t < STAGES - 1; ++t) {
    for (int q = 0; q < 4; ++q) issue(t, q);
    advance();
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);
  lds_barrier();
  frags(a0, b0, (const lds_byte_t*)lds, 0);
  int cur = 0;
  for (int it = 0; it < p.iters; ++it) {
    const lds_byte_t* st = (const lds_byte_t*)lds + cur * kStage;
    const int nxt = cur + 1 == STAGES ? 0 : cur + 1;
    const int fill_stage = cur == 0 ? STAGES - 1 : cur - 1;
    frags(a1, b1, st, 1);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int c = 0; c < 2; ++c) acc[i][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b0[c], a0[i], acc[i][c], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      issue(fill_stage, i);
    }
    advance();
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(0x0F78);      // vmcnt(8): the next tile has landed, two younger (four loads each) in flight
    lds_barrier();
    frags(a0, b0, (const lds_byte_t*)lds + nxt * kStage, 0);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int c = 0; c < 2; ++c) acc[i][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b1[c], a1[i], acc[i][c], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    cur = nxt;
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);
  __syncthreads();
  float s = 0.f;
  for (int i = 0; i < 4; ++i) for (int c = 0; c < 2; ++c) for (int q = 0; q < 16; ++q) s += acc[i][c][q];
  if (s == 123.456f) p.out[threadIdx.x] = s;
}

// ---- F: E on v_mfma_f32_16x16x32_bf16 ---------------------------------------------------------------------------
// The wave's 128 x 64 block as 8 x 4 tiles of 16 x 16.  A K tile in two halves: row blocks 0, 1 (a0: four 16-row
// fragments), then 2, 3 (a1), each against four 16-column fragments b that are read once per tile and replaced by the
// next tile's one by one as the second half is done with them.
template <bool BARRIER, bool LOADS, bool READS>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2))) void loop_256x256_8waves_16(const LoopArgs p) {
  constexpr int kStage = 32768, STAGES = 4;
  __shared__ __attribute__((aligned(1024))) unsigned char lds[STAGES * kStage];
  for (int i = threadIdx.x; i < STAGES * kStage / 4; i += 512) ((uint32_t*)lds)[i] = 0x3e003e00u;
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, wm = (wave >> 1) & 1, wn = wave & 1, hh = wave >> 2;
  const int x = blockIdx.x % 8, j = blockIdx.x / 8;
  const unsigned char* gp = p.g + ((size_t)x * (32 / p.share) + (j % 32) / p.share) * p.window + threadIdx.x * 16;
  size_t goff = ((size_t)(j % p.share) * 65536) % p.window;
  if (goff + kStage > p.window) goff = 0;
  f32x16 acc[4][2];
  for (int i = 0; i < 4; ++i) for (int c = 0; c < 2; ++c) for (int q = 0; q < 16; ++q) acc[i][c][q] = 0.f;
  bf16x8 a0[4], a1[4], b[4];
  const int la = dma_off16(lane & 15, lane >> 4) + wm * 2048, lb = 16384 + dma_off16(lane & 15, lane >> 4) + (wn * 4 + hh * 2) * 2048;
  auto rows = [&](bf16x8 (&a)[4], const lds_byte_t* st, int half) {
#pragma unroll
    for (int q = 0; q < 4; ++q)
      a[q] = *(const __attribute__((address_space(3))) bf16x8*)(st + la + (2 * half + (q >> 1)) * 4096 + (q & 1) * 1024);
  };
  auto col = [&](const lds_byte_t* st, int q) {
    b[q] = *(const __attribute__((address_space(3))) bf16x8*)(st + lb + (q >> 1) * 2048 + (q & 1) * 1024);
  };
  auto group = [&](const bf16x8 (&a)[4], int half, int q) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      f32x16& t = acc[2 * half + (r >> 1)][q >> 1];
      const int e = 4 * (2 * (r & 1) + (q & 1));
      f32x4 c = {t[e], t[e + 1], t[e + 2], t[e + 3]};
      c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b[q], a[r], c, 0, 0, 0);
      t[e] = c[0]; t[e + 1] = c[1]; t[e + 2] = c[2]; t[e + 3] = c[3];
    }
  };
  const unsigned lds0 = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)(lds_byte_t*)lds);
  const unsigned wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  auto issue = [&](int stage, int q) {
    const unsigned char* src = gp + goff + q * 8192;
    DMA(src, lds0 + stage * kStage + q * 8192 + wv * 1024);
  };
  auto advance = [&]() {
    goff += kStage;
    if (goff + kStage > p.window) goff = 0;
  };
  for (int t = 0; t < STAGES - 1; ++t) {
    for (int q = 0; q < 4; ++q) issue(t, q);
    advance();
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);
  lds_barrier();
  rows(a0, (const lds_byte_t*)lds, 0);
  for (int q = 0; q < 4; ++q) col((const lds_byte_t*)lds, q);
  int cur = 0;
  for (int it = 0; it < p.iters; ++it) {
    const lds_byte_t* st = (const lds_byte_t*)lds + cur * kStage;
    const int nxt = cur + 1 == STAGES ? 0 : cur + 1;
    const int fill_stage = cur == 0 ? STAGES - 1 : cur - 1;
    if (READS || it == 0) rows(a1, st, 1);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      __builtin_amdgcn_sched_barrier(0);
      group(a0, 0, q);
      __builtin_amdgcn_sched_barrier(0);
      if (LOADS) issue(fill_stage, q);
    }
    advance();
    __builtin_amdgcn_sched_barrier(0);
    if (LOADS) __builtin_amdgcn_s_waitcnt(0x0F78);      // vmcnt(8): the next tile has landed, two younger (four loads each) in flight
    if (BARRIER) lds_barrier();
    const lds_byte_t* sn = (const lds_byte_t*)lds + nxt * kStage;
    if (READS) rows(a0, sn, 0);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      __builtin_amdgcn_sched_barrier(0);
      group(a1, 1, q);
      if (READS) col(sn, q);
      __builtin_amdgcn_sched_barrier(0);
    }
    cur = nxt;
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);
  __syncthreads();
  float s = 0.f;
  for (int i = 0; i < 4; ++i) for (int c = 0; c < 2; ++c) for (int q = 0; q < 16; ++q) s += acc[i][c][q];
  if (s == 123.456f) p.out[threadIdx.x] = s;
}

// ---- host ---------------------------------------------------------------------------------------------------
template <typename Launch>
static int timed(const char* name, double flops, Launch launch) {
  hipEvent_t e0, e1;
  CHECK(hipEventCreate(&e0));
  CHECK(hipEventCreate(&e1));
  launch(64);
  CHECK(hipDeviceSynchronize());
  float best = 0.f;
  for (int rep = 0; rep < 3; ++rep) {
    CHECK(hipEventRecord(e0));
    launch(0);
    CHECK(hipEventRecord(e1));
    CHECK(hipDeviceSynchronize());
    float ms;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    if (rep == 0 || ms < best) best = ms;
  }
  printf("%-86s %8.3f ms %8.1f TFLOP/s\n", name, best, flops / best / 1e9);
  fflush(stdout);
  return 0;
}

int main() {
  float* out;
  CHECK(hipMalloc(&out, 4096));
  unsigned char* g;
  const size_t gbytes = (size_t)1 << 30;
  CHECK(hipMalloc(&g, gbytes));
  char name[160];
  for (int random = 0; random < 2; ++random) {
    const char* tag = random ? "random operands" : "constant operands";
    hipLaunchKernelGGL(fill_kernel, dim3(4096), dim3(256), 0, 0, (uint32_t*)g, gbytes / 4, random);
    CHECK(hipDeviceSynchronize());
    const int mi = 60000;
    snprintf(name, sizeof name, "A  MFMA only 32x32x16, %s", tag);
    if (timed(name, 256.0 * 4 * mi * 32 * 32768.0, [&](int w) { hipLaunchKernelGGL(mfma_only<32>, dim3(256), dim3(256), 0, 0, out, w ? w : mi, random); })) return 1;
    snprintf(name, sizeof name, "A  MFMA only 16x16x32, %s", tag);
    if (timed(name, 256.0 * 4 * mi * 32 * 32768.0, [&](int w) { hipLaunchKernelGGL(mfma_only<16>, dim3(256), dim3(256), 0, 0, out, w ? w : mi, random); })) return 1;
    const int li = 16384;
    for (int share : {32, 16, 8, 4, 2}) {
      LoopArgs p{out, g, li, share, gbytes / (8 * (32 / share))};
      snprintf(name, sizeof name, "B  K loop, contiguous loads, %2d workgroups per stream (L2 miss share 1/%d), %s", share, share, tag);
      if (timed(name, 256.0 * 4 * li * 32 * 32768.0, [&](int w) { LoopArgs q = p; if (w) q.iters = w; hipLaunchKernelGGL(loop_256x256<0>, dim3(256), dim3(256), 0, 0, q); })) return 1;
    }
    const LoopArgs pr{out, g, li, 32, gbytes / 8};
    snprintf(name, sizeof name, "C  K loop, row-major operands (16 KB pitch), 64 B of 16 rows per load, %s", tag);
    if (timed(name, 256.0 * 4 * li * 32 * 32768.0, [&](int w) { LoopArgs q = pr; if (w) q.iters = w; hipLaunchKernelGGL(loop_256x256<1>, dim3(256), dim3(256), 0, 0, q); })) return 1;
    snprintf(name, sizeof name, "C  K loop, row-major operands (16 KB pitch), 128 B of 8 rows per load, %s", tag);
    if (timed(name, 256.0 * 4 * li * 32 * 32768.0, [&](int w) { LoopArgs q = pr; if (w) q.iters = w; hipLaunchKernelGGL(loop_256x256<2>, dim3(256), dim3(256), 0, 0, q); })) return 1;
    snprintf(name, sizeof name, "D  K loop, 256 x 128 tiles, two workgroups per compute unit, contiguous loads, %s", tag);
    if (timed(name, 512.0 * 4 * li * 16 * 32768.0, [&](int w) { LoopArgs q = pr; if (w) q.iters = w; hipLaunchKernelGGL(loop_256x128<0>, dim3(512), dim3(256), 0, 0, q); })) return 1;
    for (int share : {32, 4}) {
      LoopArgs pe{out, g, li, share, gbytes / (8 * (32 / share))};
      snprintf(name, sizeof name, "E  K loop, 256 x 256 tile on eight waves, contiguous loads, L2 miss share 1/%d, %s", share, tag);
      if (timed(name, 256.0 * 4 * li * 32 * 32768.0, [&](int w) { LoopArgs q = pe; if (w) q.iters = w; hipLaunchKernelGGL(loop_256x256_8waves, dim3(256), dim3(512), 0, 0, q); })) return 1;
    }
    for (int share : {32, 4}) {
      LoopArgs pe{out, g, li, share, gbytes / (8 * (32 / share))};
      auto variant = [&](const char* what, auto kernel) {
        snprintf(name, sizeof name, "F  K loop, eight waves, 16x16x32 instruction, L2 miss share 1/%d, %s, %s", share, what, tag);
        return timed(name, 256.0 * 4 * li * 32 * 32768.0, [&](int w) { LoopArgs q = pe; if (w) q.iters = w; hipLaunchKernelGGL(kernel, dim3(256), dim3(512), 0, 0, q); });
      };
      if (variant("whole loop", loop_256x256_8waves_16<true, true, true>)) return 1;
      if (variant("no barrier", loop_256x256_8waves_16<false, true, true>)) return 1;
      if (variant("no direct loads", loop_256x256_8waves_16<true, false, true>)) return 1;
      if (variant("no LDS reads", loop_256x256_8waves_16<true, true, false>)) return 1;
      if (variant("MFMA and loop control only", loop_256x256_8waves_16<false, false, false>)) return 1;
    }
    snprintf(name, sizeof name, "D  K loop, 256 x 128 tiles, two workgroups per compute unit, row-major operands, %s", tag);
    if (timed(name, 512.0 * 4 * li * 16 * 32768.0, [&](int w) { LoopArgs q = pr; if (w) q.iters = w; hipLaunchKernelGGL(loop_256x128<1>, dim3(512), dim3(256), 0, 0, q); })) return 1;
  }
  return 0;
}
