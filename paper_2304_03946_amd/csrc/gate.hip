// Top-k gate (paper Eq. 3): logits l = x . W_g, keep the k largest per token, softmax over them.
//
// bf16 path: HBM-bound streaming of x.  The logits come from MFMA so that the 2*d*E flops per
// token do not cap the kernel below the memory roofline: the gate weights act as the MFMA
// row operand (32 experts per tile) and 32 tokens as the column operand, hence after the
// K loop every lane holds half of one token's logits and its partner lane (lane ^ 32) the
// other half -- the top-k selection is a register scan plus one cross-lane exchange per pick.
// Both operands are read straight from global memory into the MFMA register layout; the
// contraction index is permuted identically on both sides so that each lane reads 64
// contiguous bytes of its row per 64-wide K chunk.  W_g is first transposed to [E_pad, d]
// in the workspace (tiny, stays in L2).
//
// fp32 path (small correctness configuration): one wavefront per token, sequential fp32 FMA
// per logit, wave-wide butterfly arg-max per pick.
#include "common.h"

namespace flexmoe {

constexpr int kGateThreads = 256;
constexpr float kNegInf = -__builtin_huge_valf();

static int gate_epad(int E) { return (int)align_up((size_t)E, 32); }

size_t gate_ws_bytes(int d, int E, int dtype) {
  if (dtype != FLEXMOE_BF16) return 0;
  int nt = 1;
  while (nt * 32 < E) nt <<= 1;
  return align_up((size_t)nt * 32 * d * sizeof(bf16_t), 256);
}

__global__ void gate_transpose_wg_kernel(const bf16_t* __restrict__ wg, int d, int E, int epad,
                                         bf16_t* __restrict__ wgt) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;   // feature
  const int e = blockIdx.y;                              // expert row of the transposed copy
  if (i < d && e < epad) wgt[(size_t)e * d + i] = (e < E) ? wg[(size_t)i * E + e] : (bf16_t)0;
}

union Frag {
  uint4 u;
  bf16x8 v;
};

template <int NT>   // NT tiles of 32 experts
__global__ __launch_bounds__(kGateThreads) void gate_bf16_kernel(const bf16_t* __restrict__ x,
                                                                 const bf16_t* __restrict__ wgt, int N, int d,
                                                                 int E, int k, int32_t* __restrict__ topk_idx,
                                                                 float* __restrict__ topk_w) {
  const int lane = threadIdx.x % kWave;
  const int j = lane & 31, h = lane >> 5;
  const int group = blockIdx.x * (kGateThreads / kWave) + threadIdx.x / kWave;
  const int t0 = group * 32;
  if (t0 >= N) return;                       // wave-uniform
  const int t = t0 + j;
  const int tl = min(t, N - 1);              // clamp loads of the ragged last group

  f32x16 acc[NT];
#pragma unroll
  for (int r = 0; r < NT; ++r)
#pragma unroll
    for (int n = 0; n < 16; ++n) acc[r][n] = 0.f;

  const bf16_t* xrow = x + (size_t)tl * d + 32 * h;
  const bf16_t* wrow = wgt + (size_t)j * d + 32 * h;
  const int full = d / 64;
  for (int c = 0; c < full; ++c) {
    Frag xb[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) xb[s].u = *(const uint4*)(xrow + c * 64 + s * 8);
#pragma unroll
    for (int r = 0; r < NT; ++r) {
      Frag wa[4];
#pragma unroll
      for (int s = 0; s < 4; ++s) wa[s].u = *(const uint4*)(wrow + (size_t)r * 32 * d + c * 64 + s * 8);
#pragma unroll
      for (int s = 0; s < 4; ++s) acc[r] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wa[s].v, xb[s].v, acc[r], 0, 0, 0);
    }
  }
  if (full * 64 < d) {                        // ragged K tail, 8-element pieces past d read as zero
    const int c = full;
    Frag xb[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const bool ok = c * 64 + 32 * h + s * 8 < d;
      xb[s].u = ok ? *(const uint4*)(xrow + c * 64 + s * 8) : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int r = 0; r < NT; ++r) {
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const bool ok = c * 64 + 32 * h + s * 8 < d;
        Frag wa;
        wa.u = ok ? *(const uint4*)(wrow + (size_t)r * 32 * d + c * 64 + s * 8) : make_uint4(0, 0, 0, 0);
        acc[r] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wa.v, xb[s].v, acc[r], 0, 0, 0);
      }
    }
  }

  // lane holds, for token t, the logits of experts r*32 + 8*(n/4) + 4*h + n%4
#pragma unroll
  for (int r = 0; r < NT; ++r)
#pragma unroll
    for (int n = 0; n < 16; ++n)
      if (r * 32 + 8 * (n / 4) + 4 * h + (n % 4) >= E) acc[r][n] = kNegInf;

  float sel_v[FLEXMOE_MAX_TOPK];
  int sel_e[FLEXMOE_MAX_TOPK];
#pragma unroll
  for (int p = 0; p < FLEXMOE_MAX_TOPK; ++p) {
    sel_v[p] = kNegInf;
    sel_e[p] = 0;
    if (p < k) {
      float bv = kNegInf;
      int be = 0x7fffffff;
#pragma unroll
      for (int r = 0; r < NT; ++r)
#pragma unroll
        for (int n = 0; n < 16; ++n) {          // ascending expert id: strict > keeps the lowest id on ties
          const int e = r * 32 + 8 * (n / 4) + 4 * h + (n % 4);
          if (acc[r][n] > bv) {
            bv = acc[r][n];
            be = e;
          }
        }
      const float ov = __shfl_xor(bv, 32);
      const int oe = __shfl_xor(be, 32);
      const bool mine = (bv > ov) || (bv == ov && be < oe);
      const float wv = mine ? bv : ov;
      const int we = mine ? be : oe;
#pragma unroll
      for (int r = 0; r < NT; ++r)
#pragma unroll
        for (int n = 0; n < 16; ++n)
          if (r * 32 + 8 * (n / 4) + 4 * h + (n % 4) == we) acc[r][n] = kNegInf;
      sel_v[p] = wv;
      sel_e[p] = we;
    }
  }
  if (h == 0 && t < N) {
    float ex[FLEXMOE_MAX_TOPK];
    float sum = 0.f;
#pragma unroll
    for (int p = 0; p < FLEXMOE_MAX_TOPK; ++p) {
      ex[p] = (p < k) ? expf(sel_v[p] - sel_v[0]) : 0.f;
      sum += ex[p];
    }
    const float inv = 1.f / sum;
#pragma unroll
    for (int p = 0; p < FLEXMOE_MAX_TOPK; ++p)
      if (p < k) {
        topk_idx[(size_t)t * k + p] = sel_e[p];
        topk_w[(size_t)t * k + p] = ex[p] * inv;
      }
  }
}

// fp32: one wave per token; lane owns experts lane, lane+64, ...
__global__ __launch_bounds__(kGateThreads) void gate_f32_kernel(const float* __restrict__ x,
                                                                const float* __restrict__ wg, int N, int d, int E,
                                                                int k, int32_t* __restrict__ topk_idx,
                                                                float* __restrict__ topk_w) {
  const int lane = threadIdx.x % kWave;
  const int t = blockIdx.x * (kGateThreads / kWave) + threadIdx.x / kWave;
  if (t >= N) return;
  constexpr int PER = FLEXMOE_MAX_EXPERTS / kWave;
  float l[PER];
#pragma unroll
  for (int q = 0; q < PER; ++q) l[q] = 0.f;
  const float* xr = x + (size_t)t * d;
  for (int i = 0; i < d; ++i) {
    const float xv = xr[i];
#pragma unroll
    for (int q = 0; q < PER; ++q) {
      const int e = lane + q * kWave;
      if (e < E) l[q] = fmaf(xv, wg[(size_t)i * E + e], l[q]);
    }
  }
#pragma unroll
  for (int q = 0; q < PER; ++q)
    if (lane + q * kWave >= E) l[q] = kNegInf;

  float sel_v[FLEXMOE_MAX_TOPK];
  int sel_e[FLEXMOE_MAX_TOPK];
#pragma unroll
  for (int p = 0; p < FLEXMOE_MAX_TOPK; ++p) {
    sel_v[p] = kNegInf;
    sel_e[p] = 0;
    if (p < k) {
      float bv = kNegInf;
      int be = 0x7fffffff;
#pragma unroll
      for (int q = 0; q < PER; ++q)
        if (l[q] > bv) {
          bv = l[q];
          be = lane + q * kWave;
        }
#pragma unroll
      for (int o = 32; o >= 1; o >>= 1) {
        const float ov = __shfl_xor(bv, o);
        const int oe = __shfl_xor(be, o);
        if (ov > bv || (ov == bv && oe < be)) {
          bv = ov;
          be = oe;
        }
      }
#pragma unroll
      for (int q = 0; q < PER; ++q)
        if (lane + q * kWave == be) l[q] = kNegInf;
      sel_v[p] = bv;
      sel_e[p] = be;
    }
  }
  if (lane == 0) {
    float ex[FLEXMOE_MAX_TOPK];
    float sum = 0.f;
#pragma unroll
    for (int p = 0; p < FLEXMOE_MAX_TOPK; ++p) {
      ex[p] = (p < k) ? expf(sel_v[p] - sel_v[0]) : 0.f;
      sum += ex[p];
    }
    const float inv = 1.f / sum;
#pragma unroll
    for (int p = 0; p < FLEXMOE_MAX_TOPK; ++p)
      if (p < k) {
        topk_idx[(size_t)t * k + p] = sel_e[p];
        topk_w[(size_t)t * k + p] = ex[p] * inv;
      }
  }
}

hipError_t launch_gate(const void* x, const void* wg, int N, int d, int E, int k, int dtype, int32_t* idx, float* w,
                       void* ws, hipStream_t s) {
  if (N == 0) return hipSuccess;
  const int wpb = kGateThreads / kWave;
  if (dtype == FLEXMOE_F32) {
    hipLaunchKernelGGL(gate_f32_kernel, dim3((N + wpb - 1) / wpb), dim3(kGateThreads), 0, s, (const float*)x,
                       (const float*)wg, N, d, E, k, idx, w);
    return hipGetLastError();
  }
  int nt = 1;
  while (nt * 32 < E) nt <<= 1;
  const int epad = nt * 32;
  bf16_t* wgt = (bf16_t*)ws;
  hipLaunchKernelGGL(gate_transpose_wg_kernel, dim3((d + 255) / 256, epad), dim3(256), 0, s, (const bf16_t*)wg, d, E,
                     epad, wgt);
  const int groups = (N + 31) / 32;
  const dim3 grid((groups + wpb - 1) / wpb), block(kGateThreads);
  const bf16_t* xb = (const bf16_t*)x;
  switch (nt) {
    case 1: hipLaunchKernelGGL(gate_bf16_kernel<1>, grid, block, 0, s, xb, wgt, N, d, E, k, idx, w); break;
    case 2: hipLaunchKernelGGL(gate_bf16_kernel<2>, grid, block, 0, s, xb, wgt, N, d, E, k, idx, w); break;
    case 4: hipLaunchKernelGGL(gate_bf16_kernel<4>, grid, block, 0, s, xb, wgt, N, d, E, k, idx, w); break;
    default: hipLaunchKernelGGL(gate_bf16_kernel<8>, grid, block, 0, s, xb, wgt, N, d, E, k, idx, w); break;
  }
  return hipGetLastError();
}

}  // namespace flexmoe
