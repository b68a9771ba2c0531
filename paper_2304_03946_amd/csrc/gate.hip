// Top-k gate (paper Eq. 3): logits l = x . W_g, keep the k largest per token, softmax over them.
//
// bf16 path: HBM-bound streaming of x.  The logits come from MFMA so that the 2*d*E flops per
// token do not cap the kernel below the memory roofline: the gate weights act as the MFMA
// row operand (32 experts per tile) and 32 tokens as the column operand, hence after the
// K loop every lane holds half of one token's logits and its partner lane (lane ^ 32) the
// other half -- the top-k selection is a register scan plus one cross-lane exchange per pick.
// W_g is first transposed to [E_pad, d_pad] in the workspace (tiny, stays in L2), except in the
// small-batch kernel with up to 64 experts, which gathers its fragments from W_g as stored.
// Large batches with up to 64 experts (gate_dma_kernel): every wave owns 32 tokens and the whole contraction; x and
// W_g^T travel global -> LDS with direct loads that fetch whole 128-byte lines of a row (eight
// rows per instruction), several 64-wide K tiles in flight per workgroup, and the MFMA fragments
// are read from LDS.  Otherwise (gate_bf16_kernel): one workgroup per 32 tokens, operands read
// straight into the MFMA register layout, the contraction split over the four waves and the
// partial logits summed in a fixed order through LDS.
//
// fp32 path (small correctness configuration): one wavefront per token, sequential fp32 FMA
// per logit, wave-wide butterfly arg-max per pick.
#include "common.h"

namespace flexmoe {

constexpr int kGateThreads = 256;
constexpr float kNegInf = -__builtin_huge_valf();

static int gate_epad(int E) { return (int)align_up((size_t)E, 32); }

constexpr int kGateDK = 64;                          // K tile of the direct-to-LDS gate kernel
static int gate_dpad(int d) { return (int)align_up((size_t)d, kGateDK); }

size_t gate_ws_bytes(int d, int E, int dtype) {
  if (dtype != FLEXMOE_BF16) return 0;
  int nt = 1;
  while (nt * 32 < E) nt <<= 1;
  return align_up((size_t)nt * 32 * gate_dpad(d) * sizeof(bf16_t), 256);
}

// wgt[e, i] = wg[i, e] for e < E, i < d; zero in the padding (rows up to epad, columns up to ld)
__global__ void gate_transpose_wg_kernel(const bf16_t* __restrict__ wg, int d, int E, int epad, int ld,
                                         bf16_t* __restrict__ wgt) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;   // feature
  const int e = blockIdx.y;                              // expert row of the transposed copy
  if (i < ld && e < epad) wgt[(size_t)e * ld + i] = (e < E && i < d) ? wg[(size_t)i * E + e] : (bf16_t)0;
}

union Frag {
  uint4 u;
  bf16x8 v;
  bf16_t h[8];
};

// Top-k selection and softmax for one tile of 32 tokens whose logits sit in MFMA layout:
// lane (j = lane%32, h = lane/32) holds, for token j, experts r*32 + 8*(n/4) + 4*h + n%4.
template <int NT>
__device__ __forceinline__ void gate_select_store(f32x16 (&acc)[NT], int t, int N, int E, int k,
                                                  int32_t* __restrict__ topk_idx, float* __restrict__ topk_w) {
  const int h = (threadIdx.x % kWave) >> 5;
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

// One workgroup = 32*CT tokens (CT = 1 in every launch).  The contraction is split over the four wavefronts (wave w takes
// the 64-wide K chunks w, w+4, ...), so even a small batch puts four waves on every compute
// unit and each wave keeps two chunks of loads in flight; the partial logits are then added in
// a fixed order (3, 2, 1, 0) through LDS, so results do not depend on timing, and wave 0 selects.
// DIRECT: `wgt` is W_g itself, [d, E]: a lane gathers the eight values of a fragment with 2-byte
// loads (stride E) instead of reading a transposed copy -- 32 NT small loads per chunk from a
// matrix that sits in L2, which saves the launch that writes the copy.  Lanes of experts >= E
// re-read expert E-1 (their logits are discarded) and rows past d re-read row d-1 (x is zero there).
template <int NT, int CT, bool DIRECT>   // NT tiles of 32 experts, CT tiles of 32 tokens
__global__ __launch_bounds__(kGateThreads) void gate_bf16_kernel(const bf16_t* __restrict__ x,
                                                                 const bf16_t* __restrict__ wgt, int N, int d,
                                                                 int E, int k, int32_t* __restrict__ topk_idx,
                                                                 float* __restrict__ topk_w) {
  __shared__ float4 partial[NT * CT * 4 * kWave];
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int j = lane & 31, h = lane >> 5;
  const int t0 = blockIdx.x * (32 * CT);

  f32x16 acc[CT][NT];
#pragma unroll
  for (int ct = 0; ct < CT; ++ct)
#pragma unroll
    for (int r = 0; r < NT; ++r)
#pragma unroll
      for (int n = 0; n < 16; ++n) acc[ct][r][n] = 0.f;

  const bf16_t* xrow[CT];
#pragma unroll
  for (int ct = 0; ct < CT; ++ct) xrow[ct] = x + (size_t)min(t0 + ct * 32 + j, N - 1) * d + 32 * h;   // clamp the ragged last tile
  const bf16_t* wrow = wgt + (size_t)j * d + 32 * h;
  const int nchunks = (d + 63) / 64;
  // DIRECT: column of W_g for the lane's expert in tile r, at row 32 h
  const bf16_t* wcol[NT];
#pragma unroll
  for (int r = 0; r < NT; ++r) wcol[r] = wgt + (size_t)(32 * h) * E + min(r * 32 + j, E - 1);
  auto gather_w = [&](int r, int k0, bool full) -> uint4 {        // W_g[k0 + 32 h + 0..7, expert]
    Frag f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int kk = full ? k0 + i : min(k0 + i, d - 1 - 32 * h);
      f.h[i] = wcol[r][(size_t)kk * E];
    }
    return f.u;
  };

  // lane reads k = 64c + 32h + 8s .. +8 of its row for s = 0..3 (64 contiguous bytes); pieces past d are zero
  auto load_chunk = [&](int c, Frag (&xb)[CT][4], Frag (&wa)[NT][4]) {
    if (c * 64 + 64 <= d) {
#pragma unroll
      for (int ct = 0; ct < CT; ++ct)
#pragma unroll
        for (int s = 0; s < 4; ++s) xb[ct][s].u = *(const uint4*)(xrow[ct] + c * 64 + s * 8);
#pragma unroll
      for (int r = 0; r < NT; ++r)
#pragma unroll
        for (int s = 0; s < 4; ++s)
          wa[r][s].u = DIRECT ? gather_w(r, c * 64 + s * 8, true) : *(const uint4*)(wrow + (size_t)r * 32 * d + c * 64 + s * 8);
    } else {
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const bool ok = c * 64 + 32 * h + s * 8 < d;
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) xb[ct][s].u = ok ? *(const uint4*)(xrow[ct] + c * 64 + s * 8) : make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int r = 0; r < NT; ++r) {
          if (DIRECT) wa[r][s].u = gather_w(r, c * 64 + s * 8, false);
          else wa[r][s].u = ok ? *(const uint4*)(wrow + (size_t)r * 32 * d + c * 64 + s * 8) : make_uint4(0, 0, 0, 0);
        }
      }
    }
  };
  auto mma_chunk = [&](const Frag (&xb)[CT][4], const Frag (&wa)[NT][4]) {
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
      for (int r = 0; r < NT; ++r)
#pragma unroll
        for (int s = 0; s < 4; ++s)
          acc[ct][r] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wa[r][s].v, xb[ct][s].v, acc[ct][r], 0, 0, 0);
  };

  // kSets chunks of loads in flight per wave (register sets used in rotation): the kernel is bound by
  // the latency of these round trips, so with few experts (small fragments) a third set pays
  constexpr int kSets = NT <= 2 ? 3 : (NT == 8 ? 1 : 2);     // 256 experts: one set, or the fragments spill
  Frag xb[kSets][CT][4], wa[kSets][NT][4];
  int c = wave;
#pragma unroll
  for (int q = 0; q < kSets; ++q)
    if (c + 4 * q < nchunks) load_chunk(c + 4 * q, xb[q], wa[q]);
  for (; c < nchunks; c += 4 * kSets) {
#pragma unroll
    for (int q = 0; q < kSets; ++q)
      if (c + 4 * q < nchunks) {
        mma_chunk(xb[q], wa[q]);
        if (c + 4 * (q + kSets) < nchunks) load_chunk(c + 4 * (q + kSets), xb[q], wa[q]);
      }
  }

  // fixed-order sum of the four partial results: wave 3 writes, waves 2 and 1 add, wave 0 finishes
#pragma unroll
  for (int turn = 3; turn >= 1; --turn) {
    if (wave == turn) {
#pragma unroll
      for (int ct = 0; ct < CT; ++ct)
#pragma unroll
        for (int r = 0; r < NT; ++r)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            float4* slot = &partial[((ct * NT + r) * 4 + q) * kWave + lane];
            float4 v = make_float4(acc[ct][r][4 * q], acc[ct][r][4 * q + 1], acc[ct][r][4 * q + 2], acc[ct][r][4 * q + 3]);
            if (turn != 3) {
              const float4 o = *slot;
              v.x += o.x; v.y += o.y; v.z += o.z; v.w += o.w;
            }
            *slot = v;
          }
    }
    __syncthreads();
  }
  if (wave != 0) return;
#pragma unroll
  for (int ct = 0; ct < CT; ++ct) {
#pragma unroll
    for (int r = 0; r < NT; ++r)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float4 o = partial[((ct * NT + r) * 4 + q) * kWave + lane];
        acc[ct][r][4 * q] += o.x; acc[ct][r][4 * q + 1] += o.y; acc[ct][r][4 * q + 2] += o.z; acc[ct][r][4 * q + 3] += o.w;
      }
    if (t0 + ct * 32 < N) gate_select_store<NT>(acc[ct], t0 + ct * 32 + j, N, E, k, topk_idx, topk_w);
  }
}

// ---------------------------------------------------------------------------------------------
// Direct-to-LDS gate for up to 64 experts.  One workgroup = WAVES waves x 32 tokens; K tiles of 64
// through S LDS stages (x tile [32*WAVES][64], W_g^T tile [32*NT][64], rows of 128 bytes whose
// 16-byte chunks are XORed with row & 7: conflict-free fragment reads).  A direct load writes lane
// i's 16 bytes at M0 + 16*i, i.e. eight lanes fill one row, so the swizzle is applied by choosing
// which chunk of the row a lane fetches.  Chunks past d come from a row of zeros (x) or from the
// zero padding of the transposed weights; token rows past N are clamped (their results are dropped).
// ---------------------------------------------------------------------------------------------
__device__ const uint4 kGateZeroRow[8] = {};
typedef __attribute__((address_space(3))) unsigned char gate_lds_t;

// s_waitcnt vmcnt(L * tiles) only (the other counters left at "no wait"): returns once at most
// `tiles` K tiles of L direct loads each are still in flight.  The immediate must be a constant.
constexpr int gate_vmcnt_imm(int n) { return 0x0F70 | (n & 15) | ((n >> 4) << 14); }
template <int L>
__device__ __forceinline__ void gate_wait_tiles(int tiles) {   // callers keep L * tiles below 64

  switch (tiles) {
    case 0: __builtin_amdgcn_s_waitcnt(gate_vmcnt_imm(0)); break;
    case 1: __builtin_amdgcn_s_waitcnt(gate_vmcnt_imm(L)); break;
    case 2: __builtin_amdgcn_s_waitcnt(gate_vmcnt_imm(2 * L)); break;
    case 3: __builtin_amdgcn_s_waitcnt(gate_vmcnt_imm(3 * L)); break;
    case 4: __builtin_amdgcn_s_waitcnt(gate_vmcnt_imm(4 * L)); break;
    case 5: __builtin_amdgcn_s_waitcnt(gate_vmcnt_imm(5 * L)); break;
    default: __builtin_amdgcn_s_waitcnt(gate_vmcnt_imm(6 * L)); break;
  }
}

template <int NT, int WAVES, int S>
__global__ __launch_bounds__(WAVES * kWave) void gate_dma_kernel(const bf16_t* __restrict__ x,
                                                                 const bf16_t* __restrict__ wgt, int N, int d,
                                                                 int dpad, int E, int k,
                                                                 int32_t* __restrict__ topk_idx,
                                                                 float* __restrict__ topk_w) {
  constexpr int kXBytes = WAVES * 32 * 128;          // x tile
  constexpr int kWBytes = NT * 32 * 128;             // W_g^T tile
  constexpr int kStage = kXBytes + kWBytes;
  constexpr int L = 4 + (NT * 4 + WAVES - 1) / WAVES;   // direct loads per wave per K tile (x: 4, W: its share)
  static_assert(S >= 3 && S - 2 <= 6 && (S - 2) * L <= 63, "the wait count has six bits");
  __shared__ __align__(1024) unsigned char smem[S * kStage];
  const int lane = threadIdx.x % kWave, wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int j = lane & 31, h = lane >> 5;
  const int t0 = blockIdx.x * (32 * WAVES) + wave * 32;
  const int KT = dpad / kGateDK;

  // x: this wave loads its own 32 token rows: instruction q covers rows 8q .. 8q+7, lane -> (row, chunk)
  const int lrow = lane >> 3, lchunk = (lane & 7) ^ (lrow & 7);
  const bf16_t* xsrc[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) xsrc[q] = x + (size_t)min(t0 + 8 * q + lrow, N - 1) * d + lchunk * 8;
  // W: the NT*4 instructions of a tile are dealt round-robin to the waves
  constexpr int kWLoads = (NT * 4 + WAVES - 1) / WAVES;
  const bf16_t* wsrc[kWLoads];
#pragma unroll
  for (int q = 0; q < kWLoads; ++q) {
    const int instr = min(q * WAVES + wave, NT * 4 - 1);      // surplus slots repeat the last instruction (same bytes)
    wsrc[q] = wgt + (size_t)(instr * 8 + lrow) * dpad + lchunk * 8;
  }
  const bf16_t* zsrc = (const bf16_t*)kGateZeroRow + (lane & 7) * 8;
  const unsigned lds_base = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)(gate_lds_t*)smem);

  // Workgroups start their contraction at different K tiles and wrap around, so that the requests in flight on the
  // chip are not all at the same column offset of their rows (measured: -7 % on 65536 tokens x 2048 features).
  // The order of a token's sum then depends on its workgroup, i.e. on the token's index only: still reproducible.
  const int kshift = (int)((blockIdx.x * 5u) % (unsigned)KT);
  auto issue = [&](int kt) {
    const unsigned st = lds_base + (kt % S) * kStage;
    const int ktr = kt + kshift < KT ? kt + kshift : kt + kshift - KT;
    const int k0 = ktr * kGateDK;
    const bool x_ok = k0 + lchunk * 8 < d;                    // whole 16-byte chunks: d is a multiple of 8
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const bf16_t* g = x_ok ? xsrc[q] + k0 : zsrc;
      asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(st + (wave * 4 + q) * 1024) : "memory");
    }
#pragma unroll
    for (int q = 0; q < kWLoads; ++q) {
      const int instr = min(q * WAVES + wave, NT * 4 - 1);
      const bf16_t* g = wsrc[q] + k0;
      asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(st + kXBytes + instr * 1024) : "memory");
    }
  };

  f32x16 acc[NT];
#pragma unroll
  for (int r = 0; r < NT; ++r)
#pragma unroll
    for (int n = 0; n < 16; ++n) acc[r][n] = 0.f;

#pragma unroll
  for (int p = 0; p < S - 1; ++p)
    if (p < KT) issue(p);
  for (int kt = 0; kt < KT; ++kt) {
    // tile kt has landed once at most the younger tiles are still in flight
    gate_wait_tiles<L>(min(S - 2, KT - 1 - kt));
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
    if (kt + S - 1 < KT) issue(kt + S - 1);                   // into the stage every wave has just left
    const gate_lds_t* xs = (const gate_lds_t*)smem + (kt % S) * kStage + wave * 32 * 128;
    const gate_lds_t* wsm = (const gate_lds_t*)smem + (kt % S) * kStage + kXBytes;
#pragma unroll
    for (int ks = 0; ks < kGateDK / 16; ++ks) {
      const int chunk = ((2 * ks + h) ^ (j & 7)) << 4;
      Frag xb;
      xb.v = *(const __attribute__((address_space(3))) bf16x8*)(xs + j * 128 + chunk);
#pragma unroll
      for (int r = 0; r < NT; ++r) {
        Frag wa;
        wa.v = *(const __attribute__((address_space(3))) bf16x8*)(wsm + (r * 32 + j) * 128 + chunk);
        acc[r] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wa.v, xb.v, acc[r], 0, 0, 0);
      }
    }
  }
  if (t0 < N) gate_select_store<NT>(acc, t0 + j, N, E, k, topk_idx, topk_w);
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
  const bf16_t* xb = (const bf16_t*)x;
  if (nt <= 2 && N >= 32768) {
    // large batches: direct-to-LDS streaming, four waves (two below 65536 tokens) share a weight tile
    const int dpad = gate_dpad(d);
    hipLaunchKernelGGL(gate_transpose_wg_kernel, dim3((dpad + 255) / 256, epad), dim3(256), 0, s, (const bf16_t*)wg, d,
                       E, epad, dpad, wgt);
#define FLEXMOE_GATE_LAUNCH(NT_, WAVES_, S_)                                                                       \
  hipLaunchKernelGGL((gate_dma_kernel<NT_, WAVES_, S_>), dim3((N + 32 * WAVES_ - 1) / (32 * WAVES_)),                \
                     dim3(WAVES_* kWave), 0, s, xb, wgt, N, d, dpad, E, k, idx, w)
    if (N >= 65536) {
      if (nt == 1) FLEXMOE_GATE_LAUNCH(1, 4, 6);
      else FLEXMOE_GATE_LAUNCH(2, 4, 6);
    } else {
      if (nt == 1) FLEXMOE_GATE_LAUNCH(1, 2, 6);
      else FLEXMOE_GATE_LAUNCH(2, 2, 6);
    }
#undef FLEXMOE_GATE_LAUNCH
    return hipGetLastError();
  }
  // small batches (a few waves per compute unit at most) and more than 64 experts: split-K kernel
  const dim3 block(kGateThreads);
  const dim3 grid((N + 31) / 32);
  if (nt <= 2) {
    // up to 64 experts: the fragments of W_g are gathered from the matrix as stored (one launch)
    const bf16_t* wgb = (const bf16_t*)wg;
    if (nt == 1) hipLaunchKernelGGL((gate_bf16_kernel<1, 1, true>), grid, block, 0, s, xb, wgb, N, d, E, k, idx, w);
    else hipLaunchKernelGGL((gate_bf16_kernel<2, 1, true>), grid, block, 0, s, xb, wgb, N, d, E, k, idx, w);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(gate_transpose_wg_kernel, dim3((d + 255) / 256, epad), dim3(256), 0, s, (const bf16_t*)wg, d, E,
                     epad, d, wgt);
  if (nt == 4) hipLaunchKernelGGL((gate_bf16_kernel<4, 1, false>), grid, block, 0, s, xb, wgt, N, d, E, k, idx, w);
  else hipLaunchKernelGGL((gate_bf16_kernel<8, 1, false>), grid, block, 0, s, xb, wgt, N, d, E, k, idx, w);
  return hipGetLastError();
}

}  // namespace flexmoe
