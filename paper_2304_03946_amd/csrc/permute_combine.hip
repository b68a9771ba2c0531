// Expert-wise layout transformation (paper Section 4) and its reverse fused with the
// gate-weighted sum of Eq. 4.  Both are HBM-bound row gathers with coalesced 16-byte
// accesses.  A row of d elements is d/8 (bf16) or d/4 (fp32) 16-byte vectors; a group of LPR
// lanes (64, 32 or 16: the largest that leaves no lane without a vector) moves one row, VPL
// vectors per lane, so a wave works on 64/LPR rows at a time and every lane of a 768-wide
// row is busy (96 vectors = 32 lanes x 3).  All loads of a wave's rows are issued before the
// first store, and a wave takes its row sets in a grid-stride loop with the next set's index
// loads ahead of the current set's stores.  Writes are always contiguous rows (permute reads
// through `src`, combine reads through `dest`), so there is no scatter and no atomic.
#include "common.h"

namespace flexmoe {

constexpr int kRowThreads = 256;
constexpr int kRowWaves = kRowThreads / kWave;
constexpr int kMaxVpl = 4;        // vectors per lane held in registers; wider rows take several passes

// xp[p,:] = x[src[p]/k,:] * scale[src[p]]
template <typename T, bool SCALE, int LPR>
__global__ __launch_bounds__(kRowThreads) void permute_kernel(const T* __restrict__ x, const int32_t* __restrict__ src,
                                                              const float* __restrict__ scale, int A, int k, int d,
                                                              T* __restrict__ xp) {
  constexpr int VN = Vec16<T>::n;
  constexpr int RPW = kWave / LPR;                       // rows per wave and pass
  const int lane = threadIdx.x % kWave;
  const int sub = lane / LPR, l = lane % LPR;
  const int wave = blockIdx.x * kRowWaves + threadIdx.x / kWave;
  const int nwaves = gridDim.x * kRowWaves;
  const int vec_per_row = d / VN;
  for (int p0 = wave * RPW; p0 < A; p0 += nwaves * RPW) {
    const int p = p0 + sub;
    const bool live = p < A;
    const int a = live ? src[p] : 0;
    const int t = a / k;
    float sc = 1.f;
    if (SCALE && live) sc = scale[a];
    const uint4* in = (const uint4*)(x + (size_t)t * d);
    uint4* out = (uint4*)(xp + (size_t)p * d);
    for (int c0 = 0; c0 < vec_per_row; c0 += LPR * kMaxVpl) {
      // every load is issued (index clamped into the row; a row past the end re-reads row 0 of x) and pinned
      // in registers before the first store, so that up to kMaxVpl round trips per lane are in flight at once
      uint4 u[kMaxVpl];
#pragma unroll
      for (int q = 0; q < kMaxVpl; ++q) u[q] = in[min(c0 + q * LPR + l, vec_per_row - 1)];
#pragma unroll
      for (int q = 0; q < kMaxVpl; ++q) asm volatile("" : "+v"(u[q].x), "+v"(u[q].y), "+v"(u[q].z), "+v"(u[q].w));
#pragma unroll
      for (int q = 0; q < kMaxVpl; ++q) {
        const int c = c0 + q * LPR + l;
        if (live && c < vec_per_row) {
          if (SCALE) {
            float v[VN];
            Vec16<T>::unpack(u[q], v);
#pragma unroll
            for (int e = 0; e < VN; ++e) v[e] *= sc;
            u[q] = Vec16<T>::pack(v);
          }
          out[c] = u[q];
        }
      }
    }
  }
}

// y[t,:] = sum_j w[t*k+j] * yp[dest[t*k+j],:]
template <typename T, bool WEIGHTED, int LPR>
__global__ __launch_bounds__(kRowThreads) void combine_kernel(const T* __restrict__ yp, const int32_t* __restrict__ dest,
                                                              const float* __restrict__ w, int N, int k, int d,
                                                              T* __restrict__ y) {
  constexpr int VN = Vec16<T>::n;
  constexpr int RPW = kWave / LPR;
  const int lane = threadIdx.x % kWave;
  const int sub = lane / LPR, l = lane % LPR;
  const int wave = blockIdx.x * kRowWaves + threadIdx.x / kWave;
  const int nwaves = gridDim.x * kRowWaves;
  const int vec_per_row = d / VN;
  for (int t0 = wave * RPW; t0 < N; t0 += nwaves * RPW) {
    const int t = t0 + sub;
    if (t >= N) continue;
    uint4* out = (uint4*)(y + (size_t)t * d);
    for (int c0 = 0; c0 < vec_per_row; c0 += LPR * kMaxVpl) {
      float acc[kMaxVpl][VN];
#pragma unroll
      for (int q = 0; q < kMaxVpl; ++q)
#pragma unroll
        for (int e = 0; e < VN; ++e) acc[q][e] = 0.f;
      for (int j = 0; j < k; ++j) {
        const int a = t * k + j;
        const uint4* row = (const uint4*)(yp + (size_t)dest[a] * d);
        const float g = WEIGHTED ? w[a] : 1.f;
        uint4 u[kMaxVpl];
#pragma unroll
        for (int q = 0; q < kMaxVpl; ++q) u[q] = row[min(c0 + q * LPR + l, vec_per_row - 1)];
#pragma unroll
        for (int q = 0; q < kMaxVpl; ++q) {
          float v[VN];
          Vec16<T>::unpack(u[q], v);
#pragma unroll
          for (int e = 0; e < VN; ++e) acc[q][e] = fmaf(g, v[e], acc[q][e]);
        }
      }
#pragma unroll
      for (int q = 0; q < kMaxVpl; ++q) {
        const int c = c0 + q * LPR + l;
        if (c < vec_per_row) out[c] = Vec16<T>::pack(acc[q]);
      }
    }
  }
}

// lanes per row: the smallest group of 16, 32 or 64 lanes that covers a row with at most kMaxVpl vectors per lane
// (more rows per wave, the same bytes in flight per lane); wider rows take 64 lanes and several passes
static int lanes_per_row(int vec_per_row) {
  if (vec_per_row <= 16 * kMaxVpl) return 16;
  if (vec_per_row <= 32 * kMaxVpl) return 32;
  return 64;
}

static int row_grid(int rows) {
  const int want = (rows + kRowWaves - 1) / kRowWaves;
  const int cap = 256 * 8;   // eight blocks per compute unit keep enough bytes in flight
  return want < cap ? (want < 1 ? 1 : want) : cap;
}

template <typename T, int LPR>
static void launch_permute_t(const T* x, const int32_t* src, const float* scale, int A, int k, int d, T* xp, hipStream_t s) {
  const dim3 grid(row_grid((A + kWave / LPR - 1) / (kWave / LPR))), block(kRowThreads);
  if (scale) hipLaunchKernelGGL((permute_kernel<T, true, LPR>), grid, block, 0, s, x, src, scale, A, k, d, xp);
  else hipLaunchKernelGGL((permute_kernel<T, false, LPR>), grid, block, 0, s, x, src, scale, A, k, d, xp);
}
template <typename T>
static void launch_permute_lpr(const T* x, const int32_t* src, const float* scale, int A, int k, int d, T* xp, hipStream_t s) {
  switch (lanes_per_row(d / Vec16<T>::n)) {
    case 64: launch_permute_t<T, 64>(x, src, scale, A, k, d, xp, s); break;
    case 32: launch_permute_t<T, 32>(x, src, scale, A, k, d, xp, s); break;
    default: launch_permute_t<T, 16>(x, src, scale, A, k, d, xp, s); break;
  }
}

hipError_t launch_permute(const void* x, const int32_t* src, const float* scale, int A, int k, int d, int dtype,
                          void* xp, hipStream_t s) {
  if (A == 0) return hipSuccess;
  if (dtype == FLEXMOE_F32) launch_permute_lpr<float>((const float*)x, src, scale, A, k, d, (float*)xp, s);
  else launch_permute_lpr<bf16_t>((const bf16_t*)x, src, scale, A, k, d, (bf16_t*)xp, s);
  return hipGetLastError();
}

template <typename T, int LPR>
static void launch_combine_t(const T* yp, const int32_t* dest, const float* w, int N, int k, int d, T* y, hipStream_t s) {
  const dim3 grid(row_grid((N + kWave / LPR - 1) / (kWave / LPR))), block(kRowThreads);
  if (w) hipLaunchKernelGGL((combine_kernel<T, true, LPR>), grid, block, 0, s, yp, dest, w, N, k, d, y);
  else hipLaunchKernelGGL((combine_kernel<T, false, LPR>), grid, block, 0, s, yp, dest, w, N, k, d, y);
}
template <typename T>
static void launch_combine_lpr(const T* yp, const int32_t* dest, const float* w, int N, int k, int d, T* y, hipStream_t s) {
  switch (lanes_per_row(d / Vec16<T>::n)) {
    case 64: launch_combine_t<T, 64>(yp, dest, w, N, k, d, y, s); break;
    case 32: launch_combine_t<T, 32>(yp, dest, w, N, k, d, y, s); break;
    default: launch_combine_t<T, 16>(yp, dest, w, N, k, d, y, s); break;
  }
}

hipError_t launch_combine(const void* yp, const int32_t* dest, const float* w, int N, int k, int d, int dtype, void* y,
                          hipStream_t s) {
  if (N == 0) return hipSuccess;
  if (dtype == FLEXMOE_F32) launch_combine_lpr<float>((const float*)yp, dest, w, N, k, d, (float*)y, s);
  else launch_combine_lpr<bf16_t>((const bf16_t*)yp, dest, w, N, k, d, (bf16_t*)y, s);
  return hipGetLastError();
}

}  // namespace flexmoe
