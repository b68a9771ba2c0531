// fp32 expert FFN (paper Eq. 2) forward and backward per vExpert bucket.
// This is the small-configuration path (the fp32 layer is a 17 MFLOP correctness case):
// one thread per output element, sequential fp32 FMA over the contraction index, so results
// are deterministic.  The performance path is the bf16 MFMA grouped GEMM.
#include "common.h"

namespace flexmoe {

constexpr int kF32Threads = 256;

// bucket (vExpert) that holds row p: largest v with voff[v] <= p
__device__ __forceinline__ int find_bucket(const int32_t* __restrict__ voff, int V, int p) {
  int lo = 0, hi = V;   // invariant: voff[lo] <= p < voff[hi]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (voff[mid] <= p) lo = mid; else hi = mid;
  }
  return lo;
}

enum { EPI_FWD1 = 0, EPI_PLAIN = 1, EPI_DH = 2 };

// C[p, n] = sum_k In[p, k] * W_e[k, n]   (WT == false, W_e is [K, NC])
//         = sum_k In[p, k] * W_e[n, k]   (WT == true,  W_e is [NC, K])
template <bool WT, int EPI>
__global__ __launch_bounds__(kF32Threads) void rows_gemm_f32(const float* __restrict__ in, const float* __restrict__ w,
                                                             const float* __restrict__ bias,
                                                             const int32_t* __restrict__ voff,
                                                             const int32_t* __restrict__ owner, int V, int A, int K,
                                                             int NC, int act, const float* __restrict__ hpre_in,
                                                             float* __restrict__ out0, float* __restrict__ out1) {
  const size_t o = (size_t)blockIdx.x * kF32Threads + threadIdx.x;
  if (o >= (size_t)A * NC) return;
  const int p = (int)(o / NC), n = (int)(o % NC);
  const int e = owner[find_bucket(voff, V, p)];
  const float* we = w + (size_t)e * K * NC;
  const float* row = in + (size_t)p * K;
  float acc = 0.f;
  for (int kk = 0; kk < K; ++kk) acc = fmaf(row[kk], WT ? we[(size_t)n * K + kk] : we[(size_t)kk * NC + n], acc);
  if (bias) acc += bias[(size_t)e * NC + n];
  if (EPI == EPI_FWD1) {          // out0 = pre-activation (kept), out1 = activation
    if (out0) out0[o] = acc;
    out1[o] = act_apply(acc, act);
  } else if (EPI == EPI_PLAIN) {
    out0[o] = acc;
  } else {                        // out0 = dHpre, out1 = act(Hpre)
    const float z = hpre_in[o];
    out0[o] = acc * act_deriv(z, act);
    out1[o] = act_apply(z, act);
  }
}

// dW_e[m, n] = sum over the vExperts v of e (ascending v), rows p of v: L[p, m] * R[p, n]
__global__ __launch_bounds__(kF32Threads) void wgrad_f32(const float* __restrict__ L, const float* __restrict__ R,
                                                         const int32_t* __restrict__ voff,
                                                         const int32_t* __restrict__ owner, int V, int M, int NC,
                                                         float* __restrict__ dw) {
  const int e = blockIdx.y;
  const size_t o = (size_t)blockIdx.x * kF32Threads + threadIdx.x;
  if (o >= (size_t)M * NC) return;
  const int m = (int)(o / NC), n = (int)(o % NC);
  float acc = 0.f;
  for (int v = 0; v < V; ++v) {
    if (owner[v] != e) continue;
    for (int p = voff[v]; p < voff[v + 1]; ++p) acc = fmaf(L[(size_t)p * M + m], R[(size_t)p * NC + n], acc);
  }
  dw[(size_t)e * M * NC + o] = acc;
}

static dim3 elems_grid(size_t n) { return dim3((unsigned)((n + kF32Threads - 1) / kF32Threads)); }

hipError_t launch_ffn_fwd_f32(const FfnArgs& a, const void* xp, const void* w1, const void* b1, const void* w2,
                              const void* b2, void* hpre, void* h_keep, void* yp, void* ws, hipStream_t s) {
  if (a.A == 0) return hipSuccess;
  float* h = h_keep ? (float*)h_keep : (float*)ws;
  hipLaunchKernelGGL((rows_gemm_f32<false, EPI_FWD1>), elems_grid((size_t)a.A * a.f), dim3(kF32Threads), 0, s,
                     (const float*)xp, (const float*)w1, (const float*)b1, a.voff, a.owner, a.V, a.A, a.d, a.f, a.act,
                     (const float*)nullptr, (float*)hpre, h);
  hipLaunchKernelGGL((rows_gemm_f32<false, EPI_PLAIN>), elems_grid((size_t)a.A * a.d), dim3(kF32Threads), 0, s,
                     (const float*)h, (const float*)w2, (const float*)b2, a.voff, a.owner, a.V, a.A, a.f, a.d, a.act,
                     (const float*)nullptr, (float*)yp, (float*)nullptr);
  return hipGetLastError();
}

// h_kept is accepted for symmetry with the bf16 path; this reference-grade path computes act(Hpre) again all the same
// and takes the weight gradient's operand from wherever the caller says.
hipError_t launch_ffn_bwd_f32(const FfnArgs& a, const void* dyp, const void* xp, const void* hpre, const void* h_kept,
                              const void* w1, const void* w2, void* dxp, void* dw1, void* dw2, void* ws, hipStream_t s) {
  float* dhpre = (float*)ws;
  float* h = dhpre + (size_t)a.A * a.f;
  const float* h_src = h_kept ? (const float*)h_kept : h;
  if (a.A > 0) {
    // dH = dYp . W2^T (W2_e is [f, d]: contraction over its second index), fused with act'
    hipLaunchKernelGGL((rows_gemm_f32<true, EPI_DH>), elems_grid((size_t)a.A * a.f), dim3(kF32Threads), 0, s,
                       (const float*)dyp, (const float*)w2, (const float*)nullptr, a.voff, a.owner, a.V, a.A, a.d, a.f,
                       a.act, (const float*)hpre, dhpre, h);
    // dXp = dHpre . W1^T (W1_e is [d, f])
    hipLaunchKernelGGL((rows_gemm_f32<true, EPI_PLAIN>), elems_grid((size_t)a.A * a.d), dim3(kF32Threads), 0, s,
                       (const float*)dhpre, (const float*)w1, (const float*)nullptr, a.voff, a.owner, a.V, a.A, a.f,
                       a.d, a.act, (const float*)nullptr, (float*)dxp, (float*)nullptr);
  }
  hipLaunchKernelGGL(wgrad_f32, dim3(elems_grid((size_t)a.f * a.d).x, a.E), dim3(kF32Threads), 0, s, h_src,
                     (const float*)dyp, a.voff, a.owner, a.V, a.f, a.d, (float*)dw2);
  hipLaunchKernelGGL(wgrad_f32, dim3(elems_grid((size_t)a.d * a.f).x, a.E), dim3(kF32Threads), 0, s, (const float*)xp,
                     (const float*)dhpre, a.voff, a.owner, a.V, a.d, a.f, (float*)dw1);
  return hipGetLastError();
}

}  // namespace flexmoe
