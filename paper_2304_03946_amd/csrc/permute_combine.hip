// Expert-wise layout transformation (paper Section 4) and its reverse fused with the
// gate-weighted sum of Eq. 4.  Both are HBM-bound row gathers with coalesced 16-byte
// accesses: one wavefront moves one row at a time, rows are taken in a grid-stride loop,
// two rows in flight per wave.  Writes are always contiguous rows (permute reads through
// `src`, combine reads through `dest`), so there is no scatter and no atomic.
#include "common.h"

namespace flexmoe {

constexpr int kRowThreads = 256;
constexpr int kRowWaves = kRowThreads / kWave;

// xp[p,:] = x[src[p]/k,:] * scale[src[p]]
template <typename T, bool SCALE>
__global__ __launch_bounds__(kRowThreads) void permute_kernel(const T* __restrict__ x, const int32_t* __restrict__ src,
                                                              const float* __restrict__ scale, int A, int k, int d,
                                                              T* __restrict__ xp) {
  constexpr int VN = Vec16<T>::n;
  const int lane = threadIdx.x % kWave;
  const int wave = blockIdx.x * kRowWaves + threadIdx.x / kWave;
  const int nwaves = gridDim.x * kRowWaves;
  const int vec_per_row = d / VN;
  for (int p = wave; p < A; p += nwaves) {
    const int a = src[p];
    const int t = a / k;
    float sc = 1.f;
    if (SCALE) sc = scale[a];
    const uint4* in = (const uint4*)(x + (size_t)t * d);
    uint4* out = (uint4*)(xp + (size_t)p * d);
    for (int c = lane; c < vec_per_row; c += kWave) {
      uint4 u = in[c];
      if (SCALE) {
        float v[VN];
        Vec16<T>::unpack(u, v);
#pragma unroll
        for (int q = 0; q < VN; ++q) v[q] *= sc;
        u = Vec16<T>::pack(v);
      }
      out[c] = u;
    }
  }
}

// y[t,:] = sum_j w[t*k+j] * yp[dest[t*k+j],:]
template <typename T, bool WEIGHTED>
__global__ __launch_bounds__(kRowThreads) void combine_kernel(const T* __restrict__ yp, const int32_t* __restrict__ dest,
                                                              const float* __restrict__ w, int N, int k, int d,
                                                              T* __restrict__ y) {
  constexpr int VN = Vec16<T>::n;
  const int lane = threadIdx.x % kWave;
  const int wave = blockIdx.x * kRowWaves + threadIdx.x / kWave;
  const int nwaves = gridDim.x * kRowWaves;
  const int vec_per_row = d / VN;
  for (int t = wave; t < N; t += nwaves) {
    uint4* out = (uint4*)(y + (size_t)t * d);
    for (int c = lane; c < vec_per_row; c += kWave) {
      float acc[VN];
#pragma unroll
      for (int q = 0; q < VN; ++q) acc[q] = 0.f;
      for (int j = 0; j < k; ++j) {
        const int a = t * k + j;
        const uint4 u = ((const uint4*)(yp + (size_t)dest[a] * d))[c];
        const float g = WEIGHTED ? w[a] : 1.f;
        float v[VN];
        Vec16<T>::unpack(u, v);
#pragma unroll
        for (int q = 0; q < VN; ++q) acc[q] = fmaf(g, v[q], acc[q]);
      }
      out[c] = Vec16<T>::pack(acc);
    }
  }
}

static int row_grid(int rows) {
  const int want = (rows + kRowWaves - 1) / kRowWaves;
  const int cap = 256 * 8;   // eight blocks per compute unit keep enough bytes in flight
  return want < cap ? (want < 1 ? 1 : want) : cap;
}

hipError_t launch_permute(const void* x, const int32_t* src, const float* scale, int A, int k, int d, int dtype,
                          void* xp, hipStream_t s) {
  if (A == 0) return hipSuccess;
  const dim3 grid(row_grid(A)), block(kRowThreads);
  if (dtype == FLEXMOE_F32) {
    if (scale) hipLaunchKernelGGL((permute_kernel<float, true>), grid, block, 0, s, (const float*)x, src, scale, A, k, d, (float*)xp);
    else hipLaunchKernelGGL((permute_kernel<float, false>), grid, block, 0, s, (const float*)x, src, scale, A, k, d, (float*)xp);
  } else {
    if (scale) hipLaunchKernelGGL((permute_kernel<bf16_t, true>), grid, block, 0, s, (const bf16_t*)x, src, scale, A, k, d, (bf16_t*)xp);
    else hipLaunchKernelGGL((permute_kernel<bf16_t, false>), grid, block, 0, s, (const bf16_t*)x, src, scale, A, k, d, (bf16_t*)xp);
  }
  return hipGetLastError();
}

hipError_t launch_combine(const void* yp, const int32_t* dest, const float* w, int N, int k, int d, int dtype, void* y,
                          hipStream_t s) {
  if (N == 0) return hipSuccess;
  const dim3 grid(row_grid(N)), block(kRowThreads);
  if (dtype == FLEXMOE_F32) {
    if (w) hipLaunchKernelGGL((combine_kernel<float, true>), grid, block, 0, s, (const float*)yp, dest, w, N, k, d, (float*)y);
    else hipLaunchKernelGGL((combine_kernel<float, false>), grid, block, 0, s, (const float*)yp, dest, w, N, k, d, (float*)y);
  } else {
    if (w) hipLaunchKernelGGL((combine_kernel<bf16_t, true>), grid, block, 0, s, (const bf16_t*)yp, dest, w, N, k, d, (bf16_t*)y);
    else hipLaunchKernelGGL((combine_kernel<bf16_t, false>), grid, block, 0, s, (const bf16_t*)yp, dest, w, N, k, d, (bf16_t*)y);
  }
  return hipGetLastError();
}

}  // namespace flexmoe
