// flexmoe_route for callers that cannot allocate device memory or pass a workspace (code under HIP
// graph capture, tight serving loops, harnesses that forbid hipMalloc).  Same kernels as
// flexmoe_route; the per-unit expert histograms live in a file-scope device array instead of a caller
// workspace.  Every GPU holds its own copy of the array at its own address: the address is looked up
// once per device, with that device current, and kept; host code only ever uses the looked-up pointer
// (the array's name is a host-side stand-in, not a device address).
#include <atomic>

#include "common.h"

using namespace flexmoe;

static __device__ __align__(256) unsigned char scratch[FLEXMOE_ROUTE_STATIC_SCRATCH_BYTES];

// Device address of `scratch` on the current device.
static hipError_t static_scratch(void** out) {
  constexpr int kCached = 64;
  static std::atomic<void*> ptr_of_device[kCached];
  int dev = 0;
  hipError_t err = hipGetDevice(&dev);
  if (err != hipSuccess) return err;
  const bool cached = dev >= 0 && dev < kCached;
  if (cached) {
    void* p = ptr_of_device[dev].load(std::memory_order_acquire);
    if (p) {
      *out = p;
      return hipSuccess;
    }
  }
  void* p = nullptr;
  err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
  if (err != hipSuccess) return err;
  if (!p) return hipErrorInvalidSymbol;
  if (cached) ptr_of_device[dev].store(p, std::memory_order_release);
  *out = p;
  return hipSuccess;
}

extern "C" int flexmoe_route_static(const int32_t* topk_idx, int N, int k, int E, int V, const int32_t* rep_off_host,
                                    const int32_t* rep_ids_host, int32_t* expert_count, int32_t* vexpert_count,
                                    int32_t* vexpert_off, int32_t* vexpert_owner, int32_t* dest, int32_t* src,
                                    void* stream) {
  PlacementArg tab = {};
  const int st = route_check(topk_idx, N, k, E, V, rep_off_host, rep_ids_host, expert_count, vexpert_count, vexpert_off,
                             vexpert_owner, dest, src, &tab);
  if (st != FLEXMOE_OK) return st;
  const int A = N * k;
  if (route_ws_bytes(A, E) > (size_t)FLEXMOE_ROUTE_STATIC_SCRATCH_BYTES) return FLEXMOE_SCRATCH_LIMIT;
  void* ptr = nullptr;
  if (static_scratch(&ptr) != hipSuccess) return FLEXMOE_DEVICE_ERROR;
  const hipError_t err = launch_route(topk_idx, A, E, V, tab, expert_count, vexpert_count, vexpert_off, vexpert_owner,
                                      dest, src, ptr, (hipStream_t)stream);
  return err == hipSuccess ? FLEXMOE_OK : FLEXMOE_DEVICE_ERROR;
}
