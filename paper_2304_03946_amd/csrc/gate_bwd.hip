// The rest of a trainable layer: the gradient through the gate (paper Eq. 3-4) and the bias
// gradients of the expert FFN (Eq. 2).
//
//   dg[t,j] = <dY_t, Yp[dest[t*k+j]]>                          (Eq. 4 is linear in the gate values)
//   dl[t,j] = g[t,j] * (dg[t,j] - sum_i g[t,i] dg[t,i])         (softmax over the k kept logits, Eq. 3)
//   dX_t   += sum_j dl[t,j] * W_g[:, e_j]                       (logits l = x.W_g)
//   dW_g[:,e] = sum over the assignments routed to e of dl * x  (same sum, seen from the weights)
//   db2_e = sum of the rows of dYp in e's buckets, db1_e = the same for dHpre
//
// All of it is HBM-bound row traffic.  The per-expert sums run over the bucketed layout
// (an expert's rows are contiguous per vExpert), in two stages with a fixed summation order, so
// results are reproducible: no atomics.
#include "common.h"

namespace flexmoe {

constexpr int kBwdThreads = 256;
constexpr int kBwdWaves = kBwdThreads / kWave;
constexpr int kChunkRows = 128;                    // rows of one bucket summed by one workgroup
constexpr int kChunkCols = 512;                    // columns per workgroup: 64 lanes x 16 bytes of bf16

// [rows, cols] -> [cols, rows], both row-major (the gate weights are small: no tiling)
template <typename T>
__global__ __launch_bounds__(kBwdThreads) void transpose_small_kernel(const T* __restrict__ in, int rows, int cols,
                                                                      T* __restrict__ out) {
  const int n = rows * cols;
  for (int i = blockIdx.x * kBwdThreads + threadIdx.x; i < n; i += gridDim.x * kBwdThreads) {
    const int c = i / rows, r = i % rows;          // consecutive threads write consecutive outputs
    out[i] = in[(size_t)r * cols + c];
  }
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = kWave / 2; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// One wave per token: the k gate-value gradients, the logit gradients, and the gate path's
// share of dX added in place.  wgT is W_g transposed ([E, d]) so that an expert's column is a row.
template <typename T>
__global__ __launch_bounds__(kBwdThreads) void gate_bwd_token_kernel(
    const T* __restrict__ dy, const T* __restrict__ yp, const int32_t* __restrict__ dest,
    const int32_t* __restrict__ idx, const float* __restrict__ w, const T* __restrict__ wgT, int N, int k, int d,
    float* __restrict__ dl, T* __restrict__ dx) {
  constexpr int VN = Vec16<T>::n;
  const int lane = threadIdx.x % kWave;
  const int wave = blockIdx.x * kBwdWaves + threadIdx.x / kWave;
  const int nwaves = gridDim.x * kBwdWaves;
  const int vec_per_row = d / VN;
  for (int t = wave; t < N; t += nwaves) {
    const uint4* dy_row = (const uint4*)(dy + (size_t)t * d);
    float dg[FLEXMOE_MAX_TOPK], g[FLEXMOE_MAX_TOPK], dlv[FLEXMOE_MAX_TOPK];
    int e[FLEXMOE_MAX_TOPK];
    float inner = 0.f;
#pragma unroll
    for (int j = 0; j < FLEXMOE_MAX_TOPK; ++j) {
      dg[j] = 0.f;
      g[j] = 0.f;
      e[j] = 0;
      if (j < k) {
        const int a = t * k + j;
        const uint4* yp_row = (const uint4*)(yp + (size_t)dest[a] * d);
        float acc = 0.f;
        for (int c = lane; c < vec_per_row; c += kWave) {
          float u[VN], v[VN];
          Vec16<T>::unpack(dy_row[c], u);
          Vec16<T>::unpack(yp_row[c], v);
#pragma unroll
          for (int q = 0; q < VN; ++q) acc = fmaf(u[q], v[q], acc);
        }
        dg[j] = wave_sum(acc);
        g[j] = w[a];
        e[j] = idx[a];
        inner = fmaf(g[j], dg[j], inner);
      }
    }
#pragma unroll
    for (int j = 0; j < FLEXMOE_MAX_TOPK; ++j) {
      dlv[j] = g[j] * (dg[j] - inner);
      if (j < k && lane == 0) dl[t * k + j] = dlv[j];
    }
    uint4* dx_row = (uint4*)(dx + (size_t)t * d);
    for (int c = lane; c < vec_per_row; c += kWave) {
      float acc[VN];
      Vec16<T>::unpack(dx_row[c], acc);
#pragma unroll
      for (int j = 0; j < FLEXMOE_MAX_TOPK; ++j)
        if (j < k) {
          float v[VN];
          Vec16<T>::unpack(((const uint4*)(wgT + (size_t)e[j] * d))[c], v);
#pragma unroll
          for (int q = 0; q < VN; ++q) acc[q] = fmaf(dlv[j], v[q], acc[q]);
        }
      dx_row[c] = Vec16<T>::pack(acc);
    }
  }
}

// Chunks: every bucket is cut into pieces of kChunkRows rows; flat chunk ids run over the buckets
// in ascending vExpert id.  chunk_start[v] = id of bucket v's first chunk (one wave's scan).
__device__ __forceinline__ void chunk_starts(const int32_t* __restrict__ voff, int V, int* chunk_start) {
  if (threadIdx.x < kWave) {
    const int lane = threadIdx.x;
    const int per = (V + kWave - 1) / kWave;
    int cnt[FLEXMOE_MAX_VEXPERTS / kWave];
    int sum = 0;
#pragma unroll
    for (int q = 0; q < FLEXMOE_MAX_VEXPERTS / kWave; ++q) {
      const int v = lane * per + q;
      cnt[q] = 0;
      if (q < per && v < V) cnt[q] = (voff[v + 1] - voff[v] + kChunkRows - 1) / kChunkRows;
      sum += cnt[q];
    }
    int incl = sum;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
      const int up = __shfl_up(incl, o);
      if (lane >= o) incl += up;
    }
    int start = incl - sum;
#pragma unroll
    for (int q = 0; q < FLEXMOE_MAX_VEXPERTS / kWave; ++q) {
      const int v = lane * per + q;
      if (q < per && v <= V) chunk_start[v] = start;     // entry V = total number of chunks
      start += cnt[q];
    }
    if (lane == kWave - 1 && per * kWave == V) chunk_start[V] = incl;
  }
  __syncthreads();
}

// Stage 1: partial[chunk, c] = sum over the chunk's rows of weight(row) * in[row, c], fp32.
// WEIGHTED: weight(row p) = row_w[src[p]] (a value per assignment id); otherwise 1.
// Wave w sums rows w, w+4, ... of the chunk in ascending order; the four waves' sums are added
// in wave order through LDS.
template <typename T, bool WEIGHTED>
__global__ __launch_bounds__(kBwdThreads) void bucket_colsum_partial_kernel(
    const T* __restrict__ in, const float* __restrict__ row_w, const int32_t* __restrict__ src,
    const int32_t* __restrict__ voff, int V, int C, float* __restrict__ partial) {
  constexpr int VN = Vec16<T>::n;
  __shared__ int chunk_start[FLEXMOE_MAX_VEXPERTS + 1];
  __shared__ float red[kBwdWaves][kWave][VN];
  chunk_starts(voff, V, chunk_start);
  const int chunk = blockIdx.x;
  if (chunk >= chunk_start[V]) return;               // uniform
  // bucket of this chunk: the last v with chunk_start[v] <= chunk (binary search, every thread)
  int lo = 0, hi = V - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (chunk_start[mid] <= chunk) lo = mid;
    else hi = mid - 1;
  }
  const int v = lo;
  const int row0 = voff[v] + (chunk - chunk_start[v]) * kChunkRows;
  const int rows = min(kChunkRows, voff[v + 1] - row0);
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int col = blockIdx.y * kChunkCols * VN / 8 + lane * VN;      // 512 bf16 or 256 fp32 columns per block
  float acc[VN];
#pragma unroll
  for (int q = 0; q < VN; ++q) acc[q] = 0.f;
  if (col < C) {
    // eight rows in flight per wave; the sum itself stays in ascending row order
    constexpr int U = 8;
    for (int r0 = wave; r0 < rows; r0 += kBwdWaves * U) {
      uint4 raw[U];
      float wt[U];
#pragma unroll
      for (int i = 0; i < U; ++i) {
        const int r = r0 + i * kBwdWaves;
        const int p = row0 + min(r, rows - 1);
        raw[i] = *(const uint4*)(in + (size_t)p * C + col);
        wt[i] = r < rows ? (WEIGHTED ? row_w[src[p]] : 1.f) : 0.f;
      }
#pragma unroll
      for (int i = 0; i < U; ++i) {
        if (r0 + i * kBwdWaves < rows) {
          float u[VN];
          Vec16<T>::unpack(raw[i], u);
#pragma unroll
          for (int q = 0; q < VN; ++q) acc[q] = fmaf(wt[i], u[q], acc[q]);
        }
      }
    }
  }
#pragma unroll
  for (int q = 0; q < VN; ++q) red[wave][lane][q] = acc[q];
  __syncthreads();
  if (wave == 0 && col < C) {
#pragma unroll
    for (int q = 0; q < VN; ++q) {
      float s = red[0][lane][q];
      for (int ww = 1; ww < kBwdWaves; ++ww) s += red[ww][lane][q];
      partial[(size_t)chunk * C + col + q] = s;
    }
  }
}

// Stage 2: out[e, c] = sum of the partials of e's chunks.  One workgroup per (expert, 64 columns):
// the expert's chunks, numbered through its buckets in ascending vExpert id and ascending row
// order, are dealt round-robin to the four waves; each wave adds its chunks in that order (four
// loads in flight), then the waves' sums are added in wave order.  A fixed order: reproducible.
// TRANSPOSED: out is [C, E] (the gate weights' layout).
template <typename T, bool TRANSPOSED>
__global__ __launch_bounds__(kBwdThreads) void bucket_colsum_final_kernel(
    const float* __restrict__ partial, const int32_t* __restrict__ voff, const int32_t* __restrict__ owner, int V,
    int E, int C, T* __restrict__ out) {
  __shared__ int chunk_start[FLEXMOE_MAX_VEXPERTS + 1];
  __shared__ int list[FLEXMOE_MAX_VEXPERTS];          // the expert's buckets, ascending
  __shared__ int nlist;
  __shared__ float red[kBwdWaves][kWave];
  chunk_starts(voff, V, chunk_start);
  const int e = blockIdx.y;
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  {
    // ascending list of the expert's buckets: ballot compaction, two buckets per thread
    constexpr int kSeg = FLEXMOE_MAX_VEXPERTS / kWave;             // 64-bucket segments
    __shared__ int seg_count[kSeg];
    const unsigned long long lt = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    bool mine[kSeg / kBwdWaves];
    int pos[kSeg / kBwdWaves];
#pragma unroll
    for (int h = 0; h < kSeg / kBwdWaves; ++h) {
      const int v = (h * kBwdWaves + wave) * kWave + lane;
      mine[h] = v < V && owner[v] == e;
      const unsigned long long m = __ballot(mine[h]);
      pos[h] = __popcll(m & lt);
      if (lane == 0) seg_count[h * kBwdWaves + wave] = __popcll(m);
    }
    __syncthreads();
#pragma unroll
    for (int h = 0; h < kSeg / kBwdWaves; ++h) {
      const int seg = h * kBwdWaves + wave;
      int base = 0;
      for (int q = 0; q < seg; ++q) base += seg_count[q];
      if (mine[h]) list[base + pos[h]] = seg * kWave + lane;
    }
    if (threadIdx.x == 0) {
      int n = 0;
      for (int q = 0; q < kSeg; ++q) n += seg_count[q];
      nlist = n;
    }
    __syncthreads();
  }
  const int c = blockIdx.x * kWave + lane;
  float s = 0.f;
  if (c < C) {
    int ord = 0;                                       // running number of the expert's chunks
    for (int i = 0; i < nlist; ++i) {
      const int v = list[i];
      const int first = chunk_start[v], cnt = chunk_start[v + 1] - first;
      // this wave's chunks of the bucket: ordinals congruent to `wave` modulo 4
      int j = (wave - ord % kBwdWaves + kBwdWaves) % kBwdWaves;
      for (; j + 3 * kBwdWaves < cnt; j += 4 * kBwdWaves) {
        const float p0 = partial[(size_t)(first + j) * C + c];
        const float p1 = partial[(size_t)(first + j + kBwdWaves) * C + c];
        const float p2 = partial[(size_t)(first + j + 2 * kBwdWaves) * C + c];
        const float p3 = partial[(size_t)(first + j + 3 * kBwdWaves) * C + c];
        s += p0;
        s += p1;
        s += p2;
        s += p3;
      }
      for (; j < cnt; j += kBwdWaves) s += partial[(size_t)(first + j) * C + c];
      ord += cnt;
    }
  }
  red[wave][lane] = s;
  __syncthreads();
  if (wave == 0 && c < C) {
    float t = red[0][lane];
    for (int ww = 1; ww < kBwdWaves; ++ww) t += red[ww][lane];
    Elem<T>::store(out + (TRANSPOSED ? (size_t)c * E + e : (size_t)e * C + c), t);
  }
}

static int max_chunks(int A, int V) { return A / kChunkRows + V; }
static size_t partial_bytes(int A, int V, int C) { return align_up((size_t)max_chunks(A, V) * C * sizeof(float), 256); }

template <typename T, bool WEIGHTED, bool TRANSPOSED>
static hipError_t bucket_colsum(const void* in, const float* row_w, const int32_t* src, const int32_t* voff,
                                const int32_t* owner, int A, int V, int E, int C, float* partial, void* out,
                                hipStream_t s) {
  const int cols_per_block = kChunkCols * Vec16<T>::n / 8;
  const dim3 grid1(max_chunks(A, V), (C + cols_per_block - 1) / cols_per_block);
  hipLaunchKernelGGL((bucket_colsum_partial_kernel<T, WEIGHTED>), grid1, dim3(kBwdThreads), 0, s, (const T*)in, row_w,
                     src, voff, V, C, partial);
  const dim3 grid2((C + kWave - 1) / kWave, E);
  hipLaunchKernelGGL((bucket_colsum_final_kernel<T, TRANSPOSED>), grid2, dim3(kBwdThreads), 0, s, partial, voff, owner,
                     V, E, C, (T*)out);
  return hipGetLastError();
}

size_t gate_bwd_ws_bytes(int A, int d, int E, int V, int dtype) {
  const size_t s = dtype == FLEXMOE_BF16 ? 2 : 4;
  return align_up((size_t)E * d * s, 256) + partial_bytes(A, V, d);
}

template <typename T>
static hipError_t gate_bwd_t(const void* wg, const int32_t* idx, const float* w, const void* dy,
                             const void* yp, const void* xp, const int32_t* dest, const int32_t* src,
                             const int32_t* voff, const int32_t* owner, int N, int d, int E, int k, int V, float* dl,
                             void* dx, void* dwg, void* ws, hipStream_t s) {
  T* wgT = (T*)ws;
  float* partial = (float*)((char*)ws + align_up((size_t)E * d * sizeof(T), 256));
  const int A = N * k;
  if (N > 0) {
    hipLaunchKernelGGL((transpose_small_kernel<T>), dim3(min(256, (d * E + kBwdThreads - 1) / kBwdThreads)),
                       dim3(kBwdThreads), 0, s, (const T*)wg, d, E, wgT);
    const int want = (N + kBwdWaves - 1) / kBwdWaves;
    hipLaunchKernelGGL((gate_bwd_token_kernel<T>), dim3(min(want, 256 * 8)), dim3(kBwdThreads), 0, s, (const T*)dy,
                       (const T*)yp, dest, idx, w, (const T*)wgT, N, k, d, dl, (T*)dx);
  }
  // dW_g[:, e] = sum over e's bucket rows p of dl[src[p]] * Xp[p, :]
  return bucket_colsum<T, true, true>(xp, dl, src, voff, owner, A, V, E, d, partial, dwg, s);
}

hipError_t launch_gate_bwd(const void* wg, const int32_t* idx, const float* w, const void* dy,
                           const void* yp, const void* xp, const int32_t* dest, const int32_t* src,
                           const int32_t* voff, const int32_t* owner, int N, int d, int E, int k, int V, int dtype,
                           float* dl, void* dx, void* dwg, void* ws, hipStream_t s) {
  if (dtype == FLEXMOE_F32)
    return gate_bwd_t<float>(wg, idx, w, dy, yp, xp, dest, src, voff, owner, N, d, E, k, V, dl, dx, dwg, ws, s);
  return gate_bwd_t<bf16_t>(wg, idx, w, dy, yp, xp, dest, src, voff, owner, N, d, E, k, V, dl, dx, dwg, ws, s);
}

// The FFN backward leaves dHpre [A, f] at the start of its workspace; the activations behind it
// are dead once the weight gradients are done, so the partial sums go there.
size_t bias_grads_ws_bytes(int A, int d, int f, int V, int dtype) {
  const size_t s = dtype == FLEXMOE_BF16 ? 2 : 4;
  return align_up((size_t)A * f * s, 256) + partial_bytes(A, V, d > f ? d : f);
}

template <typename T>
static hipError_t bias_grads_t(const void* dyp, const int32_t* voff, const int32_t* owner, int A, int d, int f, int E,
                               int V, void* db1, void* db2, void* ws, hipStream_t s) {
  const T* dhpre = (const T*)ws;
  float* partial = (float*)((char*)ws + align_up((size_t)A * f * sizeof(T), 256));
  hipError_t err = hipSuccess;
  if (db1) err = bucket_colsum<T, false, false>(dhpre, nullptr, nullptr, voff, owner, A, V, E, f, partial, db1, s);
  if (err != hipSuccess) return err;
  if (db2) err = bucket_colsum<T, false, false>(dyp, nullptr, nullptr, voff, owner, A, V, E, d, partial, db2, s);
  return err;
}

hipError_t launch_bias_grads(const void* dyp, const int32_t* voff, const int32_t* owner, int A, int d, int f, int E,
                             int V, int dtype, void* db1, void* db2, void* ws, hipStream_t s) {
  if (dtype == FLEXMOE_F32) return bias_grads_t<float>(dyp, voff, owner, A, d, f, E, V, db1, db2, ws, s);
  return bias_grads_t<bf16_t>(dyp, voff, owner, A, d, f, E, V, db1, db2, ws, s);
}

}  // namespace flexmoe
