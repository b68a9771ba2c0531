// C ABI of libflexmoe: host-side validation and dispatch.  Nothing here allocates, frees or
// synchronises; every error is reported before any launch.
#include "common.h"

using namespace flexmoe;

namespace {

bool dtype_ok(int dtype) { return dtype == FLEXMOE_F32 || dtype == FLEXMOE_BF16; }
bool act_ok(int act) { return act == FLEXMOE_RELU || act == FLEXMOE_GELU_ERF || act == FLEXMOE_GELU_TANH; }
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int dims_status(int N, int d, int f, int E, int k, int V) {
  if (N < 0 || d < 8 || f < 8 || (d % 8) || (f % 8)) return FLEXMOE_INVALID_ARG;
  if (E < 1 || E > FLEXMOE_MAX_EXPERTS || k < 1 || k > E || k > FLEXMOE_MAX_TOPK) return FLEXMOE_INVALID_ARG;
  if (V < E || V > FLEXMOE_MAX_VEXPERTS) return FLEXMOE_INVALID_ARG;
  if ((long long)N * k >= (1ll << 30)) return FLEXMOE_INVALID_ARG;
  return FLEXMOE_OK;
}

int dev_status(hipError_t e) { return e == hipSuccess ? FLEXMOE_OK : FLEXMOE_DEVICE_ERROR; }

}  // namespace

extern "C" {

const char* flexmoe_status_str(int status) {
  switch (status) {
    case FLEXMOE_OK: return "ok";
    case FLEXMOE_INVALID_ARG: return "invalid argument";
    case FLEXMOE_BAD_PLACEMENT: return "bad placement table";
    case FLEXMOE_WORKSPACE_TOO_SMALL: return "workspace too small";
    case FLEXMOE_UNSUPPORTED: return "unsupported dtype or activation";
    case FLEXMOE_DEVICE_ERROR: return "device error";
    case FLEXMOE_SCRATCH_LIMIT: return "problem exceeds the static scratch of the allocation-free entry point";
    default: return "unknown status";
  }
}

size_t flexmoe_workspace_bytes(int N, int d, int f, int E, int k, int V, int dtype) {
  if (dims_status(N, d, f, E, k, V) != FLEXMOE_OK || !dtype_ok(dtype)) return 0;
  const int A = N * k;
  size_t need = gate_ws_bytes(d, E, dtype);
  const size_t r = route_ws_bytes(A, E);
  const size_t g = ffn_ws_bytes(A, d, f, E, V, dtype);
  const size_t gb = gate_bwd_ws_bytes(A, d, E, V, dtype);
  const size_t bg = bias_grads_ws_bytes(A, d, f, V, dtype);
  if (r > need) need = r;
  if (g > need) need = g;
  if (gb > need) need = gb;
  if (bg > need) need = bg;
  return need < 256 ? 256 : need;
}

int flexmoe_gate_topk(const void* x, const void* wg, int N, int d, int E, int k, int dtype, int32_t* topk_idx,
                      float* topk_w, void* ws, size_t ws_bytes, void* stream) {
  if (!dtype_ok(dtype)) return FLEXMOE_UNSUPPORTED;
  if (N < 0 || d < 8 || (d % 8) || E < 1 || E > FLEXMOE_MAX_EXPERTS || k < 1 || k > E || k > FLEXMOE_MAX_TOPK)
    return FLEXMOE_INVALID_ARG;
  if (N > 0 && (!x || !topk_idx || !topk_w)) return FLEXMOE_INVALID_ARG;
  if (!wg || !aligned16(x) || !aligned16(wg)) return FLEXMOE_INVALID_ARG;
  const size_t need = gate_ws_bytes(d, E, dtype);
  if (need > 0 && (!ws || !aligned16(ws))) return FLEXMOE_INVALID_ARG;
  if (ws_bytes < need) return FLEXMOE_WORKSPACE_TOO_SMALL;
  return dev_status(launch_gate(x, wg, N, d, E, k, dtype, topk_idx, topk_w, ws, (hipStream_t)stream));
}

}  // extern "C"

// Argument check of the router and conversion of the host table; shared by both router entry points.
int flexmoe::route_check(const int32_t* topk_idx, int N, int k, int E, int V, const int32_t* rep_off_host,
                       const int32_t* rep_ids_host, const int32_t* expert_count, const int32_t* vexpert_count,
                       const int32_t* vexpert_off, const int32_t* vexpert_owner, const int32_t* dest,
                       const int32_t* src, PlacementArg* tab) {
  if (N < 0 || E < 1 || E > FLEXMOE_MAX_EXPERTS || k < 1 || k > E || k > FLEXMOE_MAX_TOPK || V < E ||
      V > FLEXMOE_MAX_VEXPERTS || (long long)N * k >= (1ll << 30))
    return FLEXMOE_INVALID_ARG;
  if (!rep_off_host || !rep_ids_host || !expert_count || !vexpert_count || !vexpert_off || !vexpert_owner)
    return FLEXMOE_INVALID_ARG;
  if (N * k > 0 && (!topk_idx || !dest || !src)) return FLEXMOE_INVALID_ARG;
  // the table must partition the vExpert ids 0..V-1 into non-empty per-expert lists
  if (rep_off_host[0] != 0 || rep_off_host[E] != V) return FLEXMOE_BAD_PLACEMENT;
  for (int e = 0; e < E; ++e) {
    if (rep_off_host[e + 1] <= rep_off_host[e] || rep_off_host[e + 1] > V) return FLEXMOE_BAD_PLACEMENT;
    tab->rep_off[e] = (uint16_t)rep_off_host[e];
  }
  tab->rep_off[E] = (uint16_t)V;
  bool seen[FLEXMOE_MAX_VEXPERTS] = {false};
  for (int i = 0; i < V; ++i) {
    const int v = rep_ids_host[i];
    if (v < 0 || v >= V || seen[v]) return FLEXMOE_BAD_PLACEMENT;
    seen[v] = true;
    tab->rep_ids[i] = (uint16_t)v;
  }
  return FLEXMOE_OK;
}

extern "C" {

int flexmoe_route(const int32_t* topk_idx, int N, int k, int E, int V, const int32_t* rep_off_host,
                  const int32_t* rep_ids_host, int32_t* expert_count, int32_t* vexpert_count, int32_t* vexpert_off,
                  int32_t* vexpert_owner, int32_t* dest, int32_t* src, void* ws, size_t ws_bytes, void* stream) {
  PlacementArg tab = {};
  const int st = route_check(topk_idx, N, k, E, V, rep_off_host, rep_ids_host, expert_count, vexpert_count, vexpert_off,
                             vexpert_owner, dest, src, &tab);
  if (st != FLEXMOE_OK) return st;
  if (!ws) return FLEXMOE_INVALID_ARG;
  const int A = N * k;
  if (ws_bytes < route_ws_bytes(A, E)) return FLEXMOE_WORKSPACE_TOO_SMALL;
  return dev_status(launch_route(topk_idx, A, E, V, tab, expert_count, vexpert_count, vexpert_off, vexpert_owner,
                                 dest, src, ws, (hipStream_t)stream));
}

int flexmoe_permute(const void* x, const int32_t* src, const float* row_scale, int N, int k, int d, int dtype,
                    void* xp, void* stream) {
  if (!dtype_ok(dtype)) return FLEXMOE_UNSUPPORTED;
  if (N < 0 || k < 1 || k > FLEXMOE_MAX_TOPK || d < 8 || (d % 8) || (long long)N * k >= (1ll << 30))
    return FLEXMOE_INVALID_ARG;
  if (N > 0 && (!x || !src || !xp || !aligned16(x) || !aligned16(xp))) return FLEXMOE_INVALID_ARG;
  return dev_status(launch_permute(x, src, row_scale, N * k, k, d, dtype, xp, (hipStream_t)stream));
}

int flexmoe_combine(const void* yp, const int32_t* dest, const float* topk_w, int N, int k, int d, int dtype, void* y,
                    void* stream) {
  if (!dtype_ok(dtype)) return FLEXMOE_UNSUPPORTED;
  if (N < 0 || k < 1 || k > FLEXMOE_MAX_TOPK || d < 8 || (d % 8) || (long long)N * k >= (1ll << 30))
    return FLEXMOE_INVALID_ARG;
  if (N > 0 && (!yp || !dest || !y || !aligned16(yp) || !aligned16(y))) return FLEXMOE_INVALID_ARG;
  return dev_status(launch_combine(yp, dest, topk_w, N, k, d, dtype, y, (hipStream_t)stream));
}

static int ffn_common(int A, int d, int f, int E, int V, int act, int dtype, const void* voff, const void* owner,
                      const void* ws, size_t ws_bytes) {
  if (!dtype_ok(dtype) || !act_ok(act)) return FLEXMOE_UNSUPPORTED;
  if (A < 0 || A >= (1 << 30) || d < 8 || f < 8 || (d % 8) || (f % 8) || E < 1 || E > FLEXMOE_MAX_EXPERTS || V < E ||
      V > FLEXMOE_MAX_VEXPERTS)
    return FLEXMOE_INVALID_ARG;
  if (!voff || !owner || !ws || !aligned16(ws)) return FLEXMOE_INVALID_ARG;
  if (ws_bytes < ffn_ws_bytes(A, d, f, E, V, dtype)) return FLEXMOE_WORKSPACE_TOO_SMALL;
  return FLEXMOE_OK;
}

int flexmoe_expert_ffn_fwd(const void* xp, const int32_t* vexpert_off, const int32_t* vexpert_owner, const void* w1,
                           const void* b1, const void* w2, const void* b2, int A, int d, int f, int E, int V, int act,
                           int dtype, void* hpre, void* h, void* yp, void* ws, size_t ws_bytes, void* stream) {
  const int st = ffn_common(A, d, f, E, V, act, dtype, vexpert_off, vexpert_owner, ws, ws_bytes);
  if (st != FLEXMOE_OK) return st;
  if (!w1 || !w2 || !aligned16(w1) || !aligned16(w2) || !aligned16(b1) || !aligned16(b2)) return FLEXMOE_INVALID_ARG;
  if (A > 0 && (!xp || !yp || !aligned16(xp) || !aligned16(hpre) || !aligned16(h) || !aligned16(yp)))      // hpre, h may be NULL
    return FLEXMOE_INVALID_ARG;
  const FfnArgs a{A, d, f, E, V, act, vexpert_off, vexpert_owner};
  const hipStream_t s = (hipStream_t)stream;
  return dev_status(dtype == FLEXMOE_BF16 ? launch_ffn_fwd_bf16(a, xp, w1, b1, w2, b2, hpre, h, yp, ws, s)
                                          : launch_ffn_fwd_f32(a, xp, w1, b1, w2, b2, hpre, h, yp, ws, s));
}

int flexmoe_expert_ffn_fwd_gather(const void* x, const int32_t* src, const int32_t* vexpert_off,
                                  const int32_t* vexpert_owner, const void* w1, const void* b1, const void* w2,
                                  const void* b2, int N, int k, int d, int f, int E, int V, int act, int dtype,
                                  void* hpre, void* h, void* yp, void* ws, size_t ws_bytes, void* stream) {
  if (N < 0 || k < 1 || k > FLEXMOE_MAX_TOPK || (long long)N * k >= (1ll << 30)) return FLEXMOE_INVALID_ARG;
  const int A = N * k;
  const int st = ffn_common(A, d, f, E, V, act, dtype, vexpert_off, vexpert_owner, ws, ws_bytes);
  if (st != FLEXMOE_OK) return st;
  // gathered row loads exist on the bf16 direct-to-LDS path only; row offsets are 32-bit byte counts kept below 2^31
  if (dtype != FLEXMOE_BF16 || (d % 128) || (long long)N * d >= (1ll << 30)) return FLEXMOE_UNSUPPORTED;
  if (!w1 || !w2 || !aligned16(w1) || !aligned16(w2) || !aligned16(b1) || !aligned16(b2)) return FLEXMOE_INVALID_ARG;
  if (A > 0 && (!x || !src || !yp || !aligned16(x) || !aligned16(hpre) || !aligned16(h) || !aligned16(yp)))    // hpre, h may be NULL
    return FLEXMOE_INVALID_ARG;
  const FfnArgs a{A, d, f, E, V, act, vexpert_off, vexpert_owner};
  return dev_status(launch_ffn_fwd_gather_bf16(a, x, src, k, w1, b1, w2, b2, hpre, h, yp, ws, (hipStream_t)stream));
}

int flexmoe_expert_ffn_fwd_top1(const void* x, const int32_t* src, const int32_t* vexpert_off,
                                const int32_t* vexpert_owner, const void* w1, const void* b1, const void* w2,
                                const void* b2, int N, int d, int f, int E, int V, int act, int dtype,
                                void* hpre, void* h, void* y, void* ws, size_t ws_bytes, void* stream) {
  if (N < 0 || N >= (1 << 30)) return FLEXMOE_INVALID_ARG;
  const int st = ffn_common(N, d, f, E, V, act, dtype, vexpert_off, vexpert_owner, ws, ws_bytes);
  if (st != FLEXMOE_OK) return st;
  // gathered loads and scattered stores exist on the bf16 direct-to-LDS path only; row offsets are 32-bit byte counts kept below 2^31
  if (dtype != FLEXMOE_BF16 || (d % 128) || (f % 128) || (long long)N * d >= (1ll << 30)) return FLEXMOE_UNSUPPORTED;
  if (!w1 || !w2 || !aligned16(w1) || !aligned16(w2) || !aligned16(b1) || !aligned16(b2)) return FLEXMOE_INVALID_ARG;
  if (N > 0 && (!x || !src || !y || !aligned16(x) || !aligned16(hpre) || !aligned16(h) || !aligned16(y)))    // hpre, h may be NULL
    return FLEXMOE_INVALID_ARG;
  const FfnArgs a{N, d, f, E, V, act, vexpert_off, vexpert_owner};
  return dev_status(launch_ffn_fwd_top1_bf16(a, x, src, w1, b1, w2, b2, hpre, h, y, ws, (hipStream_t)stream));
}

int flexmoe_expert_ffn_bwd(const void* dyp, const void* xp, const void* hpre, const void* h, const void* w1, const void* w2,
                           const int32_t* vexpert_off, const int32_t* vexpert_owner, int A, int d, int f, int E, int V,
                           int act, int dtype, void* dxp, void* dw1, void* dw2, void* ws, size_t ws_bytes,
                           void* stream) {
  const int st = ffn_common(A, d, f, E, V, act, dtype, vexpert_off, vexpert_owner, ws, ws_bytes);
  if (st != FLEXMOE_OK) return st;
  if (!w1 || !w2 || !dw1 || !dw2 || !aligned16(w1) || !aligned16(w2) || !aligned16(dw1) || !aligned16(dw2))
    return FLEXMOE_INVALID_ARG;
  if (A > 0 && (!dyp || !xp || !hpre || !dxp || !aligned16(dyp) || !aligned16(xp) || !aligned16(hpre) || !aligned16(h) ||
                !aligned16(dxp)))      // h may be NULL
    return FLEXMOE_INVALID_ARG;
  const FfnArgs a{A, d, f, E, V, act, vexpert_off, vexpert_owner};
  const hipStream_t s = (hipStream_t)stream;
  return dev_status(dtype == FLEXMOE_BF16 ? launch_ffn_bwd_bf16(a, dyp, xp, hpre, h, w1, w2, dxp, dw1, dw2, ws, s)
                                          : launch_ffn_bwd_f32(a, dyp, xp, hpre, h, w1, w2, dxp, dw1, dw2, ws, s));
}

int flexmoe_expert_ffn_bwd_top1(const void* dyp, const void* xp, const void* hpre, const void* h, const void* w1, const void* w2,
                                const int32_t* vexpert_off, const int32_t* vexpert_owner, const int32_t* src,
                                int N, int d, int f, int E, int V, int act, int dtype,
                                void* dx, void* dw1, void* dw2, void* ws, size_t ws_bytes, void* stream) {
  if (N < 0 || N >= (1 << 30)) return FLEXMOE_INVALID_ARG;
  const int st = ffn_common(N, d, f, E, V, act, dtype, vexpert_off, vexpert_owner, ws, ws_bytes);
  if (st != FLEXMOE_OK) return st;
  // scattered stores exist on the bf16 direct-to-LDS path only (dXp contracts over f)
  if (dtype != FLEXMOE_BF16 || (f % 128)) return FLEXMOE_UNSUPPORTED;
  if (!w1 || !w2 || !dw1 || !dw2 || !aligned16(w1) || !aligned16(w2) || !aligned16(dw1) || !aligned16(dw2))
    return FLEXMOE_INVALID_ARG;
  if (N > 0 && (!dyp || !xp || !hpre || !dx || !src || !aligned16(dyp) || !aligned16(xp) || !aligned16(hpre) || !aligned16(h) ||
                !aligned16(dx)))      // h may be NULL
    return FLEXMOE_INVALID_ARG;
  const FfnArgs a{N, d, f, E, V, act, vexpert_off, vexpert_owner};
  return dev_status(launch_ffn_bwd_bf16(a, dyp, xp, hpre, h, w1, w2, dx, dw1, dw2, ws, (hipStream_t)stream, src));
}

int flexmoe_gate_bwd(const void* wg, const int32_t* topk_idx, const float* topk_w, const void* dy, const void* yp,
                     const void* xp, const int32_t* dest, const int32_t* src, const int32_t* vexpert_off,
                     const int32_t* vexpert_owner, int N, int d, int E, int k, int V, int dtype, float* dl, void* dx,
                     void* dwg, void* ws, size_t ws_bytes, void* stream) {
  if (!dtype_ok(dtype)) return FLEXMOE_UNSUPPORTED;
  const int st = dims_status(N, d, 8, E, k, V);
  if (st != FLEXMOE_OK) return st;
  if (!wg || !dwg || !vexpert_off || !vexpert_owner || !ws || !aligned16(wg) || !aligned16(dwg) || !aligned16(ws))
    return FLEXMOE_INVALID_ARG;
  if (N > 0 && (!topk_idx || !topk_w || !dy || !yp || !xp || !dest || !src || !dl || !dx || !aligned16(dy) ||
                !aligned16(yp) || !aligned16(xp) || !aligned16(dx)))
    return FLEXMOE_INVALID_ARG;
  if (ws_bytes < gate_bwd_ws_bytes(N * k, d, E, V, dtype)) return FLEXMOE_WORKSPACE_TOO_SMALL;
  return dev_status(launch_gate_bwd(wg, topk_idx, topk_w, dy, yp, xp, dest, src, vexpert_off, vexpert_owner, N, d, E,
                                    k, V, dtype, dl, dx, dwg, ws, (hipStream_t)stream));
}

int flexmoe_expert_bias_grads(const void* dyp, const int32_t* vexpert_off, const int32_t* vexpert_owner, int A, int d,
                              int f, int E, int V, int dtype, void* db1, void* db2, void* ws, size_t ws_bytes,
                              void* stream) {
  const int st = ffn_common(A, d, f, E, V, FLEXMOE_RELU, dtype, vexpert_off, vexpert_owner, ws, ws_bytes);
  if (st != FLEXMOE_OK) return st;
  if (!aligned16(db1) || !aligned16(db2) || (A > 0 && (!dyp || !aligned16(dyp)))) return FLEXMOE_INVALID_ARG;
  if (ws_bytes < bias_grads_ws_bytes(A, d, f, V, dtype)) return FLEXMOE_WORKSPACE_TOO_SMALL;
  return dev_status(launch_bias_grads(dyp, vexpert_off, vexpert_owner, A, d, f, E, V, dtype, db1, db2, ws,
                                      (hipStream_t)stream));
}

}  // extern "C"
