// Shared device helpers and the internal launcher interface of libflexmoe (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "flexmoe.h"

namespace flexmoe {

typedef unsigned short bf16_t;   // bf16 bit pattern
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

// fp32 -> bf16, round to nearest even (v_cvt_pk_bf16_f32 on gfx950: two values per instruction)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
__device__ __forceinline__ bf16_t f32_to_bf16(float f) { return (bf16_t)(pack_bf16x2(f, 0.f) & 0xffffu); }

template <typename T> struct Elem;
template <> struct Elem<float> {
  static __device__ __forceinline__ float load(const float* p) { return *p; }
  static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
  static __device__ __forceinline__ float load(const bf16_t* p) { return bf16_to_f32(*p); }
  static __device__ __forceinline__ void store(bf16_t* p, float v) { *p = f32_to_bf16(v); }
};

// Sixteen bytes of a row as floats (4 x fp32 or 8 x bf16) and back.
template <typename T> struct Vec16;
template <> struct Vec16<float> {
  static constexpr int n = 4;
  static __device__ __forceinline__ void unpack(const uint4& u, float* v) {
    v[0] = __uint_as_float(u.x); v[1] = __uint_as_float(u.y); v[2] = __uint_as_float(u.z); v[3] = __uint_as_float(u.w);
  }
  static __device__ __forceinline__ uint4 pack(const float* v) {
    return make_uint4(__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3]));
  }
};
template <> struct Vec16<bf16_t> {
  static constexpr int n = 8;
  static __device__ __forceinline__ void unpack(const uint4& u, float* v) {
    v[0] = __uint_as_float(u.x << 16); v[1] = __uint_as_float(u.x & 0xffff0000u);
    v[2] = __uint_as_float(u.y << 16); v[3] = __uint_as_float(u.y & 0xffff0000u);
    v[4] = __uint_as_float(u.z << 16); v[5] = __uint_as_float(u.z & 0xffff0000u);
    v[6] = __uint_as_float(u.w << 16); v[7] = __uint_as_float(u.w & 0xffff0000u);
  }
  static __device__ __forceinline__ uint4 pack(const float* v) {
    return make_uint4(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7]));
  }
};

// Activations of the expert FFN (Eq. 2 uses ReLU; GELU for the BERT/GPT/Swin-shaped layers).
// Accurate forms (libm erff/tanhf), used by the fp32 path.
__device__ __forceinline__ float act_apply(float z, int act) {
  if (act == FLEXMOE_RELU) return z > 0.f ? z : 0.f;
  if (act == FLEXMOE_GELU_ERF) return 0.5f * z * (1.f + erff(z * 0.70710678118654752f));
  const float c = 0.79788456080286536f;
  return 0.5f * z * (1.f + tanhf(c * (z + 0.044715f * z * z * z)));
}
__device__ __forceinline__ float act_deriv(float z, int act) {
  if (act == FLEXMOE_RELU) return z > 0.f ? 1.f : 0.f;
  if (act == FLEXMOE_GELU_ERF)
    return 0.5f * (1.f + erff(z * 0.70710678118654752f)) + z * 0.39894228040143268f * expf(-0.5f * z * z);
  const float c = 0.79788456080286536f;
  float u = c * (z + 0.044715f * z * z * z);
  float th = tanhf(u);
  return 0.5f * (1.f + th) + 0.5f * z * (1.f - th * th) * c * (1.f + 3.f * 0.044715f * z * z);
}

// Fast forms for the bf16 GEMM epilogues, where results are rounded to bf16 (relative 2^-9).
// The normal CDF comes from the complementary error function by the rational-exponential
// formula 7.1.26 of Abramowitz & Stegun (erfc(x) = (a1 t + ... + a5 t^5) e^{-x^2}, t = 1/(1+px),
// x >= 0, |error| <= 1.5e-7) with the hardware reciprocal (v_rcp_f32, 1 ulp) and exp2:
// Phi(-|z|) = erfc(|z|/sqrt 2)/2, Phi(|z|) = 1 - Phi(-|z|).  The same exponential e^{-z^2/2}
// gives the normal density that the GELU derivative needs.
__device__ __forceinline__ float fast_norm_cdf(float z, float* exp_neg_half_z2) {
  const float ax = fabsf(z) * 0.70710678118654752f;
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, ax, 1.f));
  float p = fmaf(0.5f * 1.061405429f, t, 0.5f * -1.453152027f);     // half the polynomial: Phi, not erfc
  p = fmaf(p, t, 0.5f * 1.421413741f);
  p = fmaf(p, t, 0.5f * -0.284496736f);
  p = fmaf(p, t, 0.5f * 0.254829592f);
  p *= t;
  const float ex = __builtin_amdgcn_exp2f(ax * ax * -1.44269504088896341f);
  *exp_neg_half_z2 = ex;
  const float q = p * ex;                                            // Phi(-|z|)
  return z > 0.f ? 1.f - q : q;
}
__device__ __forceinline__ float fast_tanh(float u) {   // 1 - 2/(1+e^{2u}), saturates cleanly
  const float e2 = __builtin_amdgcn_exp2f(fminf(u, 15.f) * 2.88539008177792681f);
  return 1.f - 2.f * __builtin_amdgcn_rcpf(e2 + 1.f);
}
template <int ACT> __device__ __forceinline__ void act_both(float z, float* a, float* da) {
  if (ACT == FLEXMOE_RELU) {
    *a = z > 0.f ? z : 0.f;
    *da = z > 0.f ? 1.f : 0.f;
  } else if (ACT == FLEXMOE_GELU_ERF) {
    float ex;
    const float cdf = fast_norm_cdf(z, &ex);
    *a = z * cdf;
    *da = fmaf(z * 0.39894228040143268f, ex, cdf);
  } else {
    const float c = 0.79788456080286536f;
    const float th = fast_tanh(c * fmaf(0.044715f * z, z * z, z));
    *a = 0.5f * z * (1.f + th);
    *da = 0.5f * (1.f + th) + 0.5f * z * (1.f - th * th) * c * fmaf(3.f * 0.044715f * z, z, 1.f);
  }
}
template <int ACT> __device__ __forceinline__ float act_fast(float z) {
  float a, da;
  act_both<ACT>(z, &a, &da);
  return a;
}

// Expert->vExpert table handed to the route kernels by value (it is a host-side input): CSR in
// uint16.  Two sizes, so that the usual layer (up to 64 experts, 128 vExperts) carries 386 bytes of
// kernel arguments instead of 1538.
template <int EMAX, int VMAX> struct PlacementArgT {
  static constexpr int kMaxExperts = EMAX, kMaxVexperts = VMAX;
  uint16_t rep_off[EMAX + 1];
  uint16_t rep_ids[VMAX];
};
typedef PlacementArgT<FLEXMOE_MAX_EXPERTS, FLEXMOE_MAX_VEXPERTS> PlacementArg;
typedef PlacementArgT<64, 128> PlacementArgSmall;

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ---- launchers (host side; each returns hipGetLastError() of its launches) ----
size_t gate_ws_bytes(int d, int E, int dtype);
hipError_t launch_gate(const void* x, const void* wg, int N, int d, int E, int k, int dtype,
                       int32_t* idx, float* w, void* ws, hipStream_t s);

// host-side argument check of the router entry points; fills the by-value table (api.hip)
int route_check(const int32_t* topk_idx, int N, int k, int E, int V, const int32_t* rep_off_host,
                const int32_t* rep_ids_host, const int32_t* expert_count, const int32_t* vexpert_count,
                const int32_t* vexpert_off, const int32_t* vexpert_owner, const int32_t* dest, const int32_t* src,
                PlacementArg* tab);
int route_units(int A, int* unit_len);
size_t route_ws_bytes(int A, int E);
hipError_t launch_route(const int32_t* idx, int A, int E, int V, const PlacementArg& tab,
                        int32_t* expert_count, int32_t* vexpert_count, int32_t* vexpert_off,
                        int32_t* vexpert_owner, int32_t* dest, int32_t* src, void* ws, hipStream_t s);

hipError_t launch_permute(const void* x, const int32_t* src, const float* scale, int A, int k, int d,
                          int dtype, void* xp, hipStream_t s);
hipError_t launch_combine(const void* yp, const int32_t* dest, const float* w, int N, int k, int d,
                          int dtype, void* y, hipStream_t s);

struct FfnArgs {
  int A, d, f, E, V, act;
  const int32_t* voff;
  const int32_t* owner;
};
size_t ffn_ws_bytes(int A, int d, int f, int E, int V, int dtype);
// h_keep / h_kept: act(Hpre) in a buffer of the caller's (written by the forward pass, read by the backward pass), or null
hipError_t launch_ffn_fwd_bf16(const FfnArgs& a, const void* xp, const void* w1, const void* b1,
                               const void* w2, const void* b2, void* hpre, void* h_keep, void* yp, void* ws, hipStream_t s);
hipError_t launch_ffn_fwd_gather_bf16(const FfnArgs& a, const void* x, const int32_t* src, int k, const void* w1,
                                      const void* b1, const void* w2, const void* b2, void* hpre, void* h_keep, void* yp,
                                      void* ws, hipStream_t s);
hipError_t launch_ffn_fwd_top1_bf16(const FfnArgs& a, const void* x, const int32_t* src, const void* w1, const void* b1,
                                    const void* w2, const void* b2, void* hpre, void* h_keep, void* y, void* ws,
                                    hipStream_t s);
hipError_t launch_ffn_bwd_bf16(const FfnArgs& a, const void* dyp, const void* xp, const void* hpre, const void* h_kept,
                               const void* w1, const void* w2, void* dxp, void* dw1, void* dw2,
                               void* ws, hipStream_t s,
                               const int32_t* scatter_src = nullptr);
// gate-path backward and bias gradients (gate_bwd.hip)
size_t gate_bwd_ws_bytes(int A, int d, int E, int V, int dtype);
hipError_t launch_gate_bwd(const void* wg, const int32_t* idx, const float* w, const void* dy,
                           const void* yp, const void* xp, const int32_t* dest, const int32_t* src,
                           const int32_t* voff, const int32_t* owner, int N, int d, int E, int k, int V, int dtype,
                           float* dl, void* dx, void* dwg, void* ws, hipStream_t s);
size_t bias_grads_ws_bytes(int A, int d, int f, int V, int dtype);
hipError_t launch_bias_grads(const void* dyp, const int32_t* voff, const int32_t* owner, int A, int d, int f, int E,
                             int V, int dtype, void* db1, void* db2, void* ws, hipStream_t s);
hipError_t launch_ffn_fwd_f32(const FfnArgs& a, const void* xp, const void* w1, const void* b1,
                              const void* w2, const void* b2, void* hpre, void* h_keep, void* yp, void* ws, hipStream_t s);
hipError_t launch_ffn_bwd_f32(const FfnArgs& a, const void* dyp, const void* xp, const void* hpre, const void* h_kept,
                              const void* w1, const void* w2, void* dxp, void* dw1, void* dw2,
                              void* ws, hipStream_t s);

}  // namespace flexmoe
