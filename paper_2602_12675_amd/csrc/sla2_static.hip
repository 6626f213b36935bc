// sla2_router_static: the router entry point for callers that cannot allocate device memory and have
// no workspace to hand over (code under graph capture, tight serving loops).  Same kernels as
// sla2_router; their intermediate arrays - fp64 block sums of Q and K, colmean(K), the folded router
// matrix - live in a file-scope device array instead of a caller's workspace.
#include <atomic>

#include "common.h"

namespace sla2 {
namespace {

static_assert(SLA2_STATIC_SCRATCH_BYTES % 256 == 0, "scratch size must keep the carve-up aligned");
static __device__ __align__(256) unsigned char scratch[SLA2_STATIC_SCRATCH_BYTES];

// Each GPU holds its own copy of the array at its own address: the address is looked up once per
// device, with that device current, and only this pointer is ever handed to a kernel (the array's name
// in host code is a host-side stand-in, not a device address).
constexpr int kMaxDevices = 64;
std::atomic<unsigned char*> g_scratch_ptr[kMaxDevices];

hipError_t scratch_of_current_device(unsigned char** out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  unsigned char* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (p == nullptr) {
    e = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (p == nullptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev].store(p, std::memory_order_release);   // two racing first calls store the same address
  }
  *out = p;
  return hipSuccess;
}

}  // namespace
}  // namespace sla2

using namespace sla2;

extern "C" int sla2_router_static(const sla2_params* params, const void* q, const void* k, const float* router_w,
                                  int32_t* block_idx, void* hip_stream) {
  Shape s; sla2_ws_layout L;
  int rc = make_shape(params, &s);
  if (rc != SLA2_OK) return rc;
  if (!q || !k || !router_w || (!block_idx && s.k > 0)) return SLA2_EINVAL;
  if (((uintptr_t)q & 15u) || ((uintptr_t)k & 15u)) return SLA2_EINVAL;
  make_layout(s, &L);
  // the router's arrays are the first ones of the workspace carve-up: [q_sum, k_sum, k_mean, router_m | block_idx ...
  const size_t need = L.block_idx;
  if (need > (size_t)SLA2_STATIC_SCRATCH_BYTES) return SLA2_EWORKSPACE;
  unsigned char* base = nullptr;
  if (scratch_of_current_device(&base) != hipSuccess) return SLA2_EHIP;
  double* q_sum = (double*)(base + L.q_sum);
  double* k_sum = (double*)(base + L.k_sum);
  double* k_mean = (double*)(base + L.k_mean);
  double* router_m = (double*)(base + L.router_m);
  hipStream_t st = (hipStream_t)hip_stream;
  // every array is written in full before it is read: nothing has to start at zero
  if (launch_block_sums(s, q, k, router_w, q_sum, k_sum, router_m, st) != hipSuccess) return SLA2_EHIP;
  if (launch_router_topk(s, q_sum, k_sum, router_m, block_idx, k_mean, st) != hipSuccess) return SLA2_EHIP;
  return SLA2_OK;
}
