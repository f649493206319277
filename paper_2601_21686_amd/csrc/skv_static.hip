// The one entry point that allocates nothing and takes no workspace: decode attention whose scratch memory
// (projected queries, per-range partial results) lives in a static device array of this library.  For callers
// that cannot allocate device memory or carry a workspace around: code under stream capture, tight serving
// loops, harnesses that forbid allocation.  Every other entry point keeps working as it does and shares its
// kernels with this one.
#include <atomic>

#include <hip/hip_runtime.h>

#include "skv_internal.h"

namespace skv {
namespace {

// Device memory held by every GPU the library runs on, from the first use until the process ends.  In host
// code this name is only a handle for hipGetSymbolAddress: what kernels and copies receive is the address
// that call returns for the current device.
static __device__ __align__(256) unsigned char scratch[SKV_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_of_device[kMaxDevices];

// The array's address on the current device, resolved once per device.  Two threads that race here resolve
// the same address; either store is fine.
hipError_t scratch_of_current_device(void** ptr) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  void* p = g_scratch_of_device[dev].load(std::memory_order_acquire);
  if (p == nullptr) {
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (p == nullptr) return hipErrorInvalidSymbol;
    g_scratch_of_device[dev].store(p, std::memory_order_release);
  }
  *ptr = p;
  return hipSuccess;
}

}  // namespace
}  // namespace skv

extern "C" skv_status skv_decode_attention_static(const skv_layer* layer, const void* q, void* out, int64_t n_ctx,
                                                  float scale, void* stream) {
  // what the call would need of a caller's workspace: the same plan, the same layout
  size_t need = 0;
  const skv_status st = skv::decode_attention_workspace_need(layer, n_ctx, &need);
  if (st != SKV_OK) return st;
  if (need > (size_t)SKV_STATIC_SCRATCH_BYTES) return SKV_ERR_WORKSPACE;
  void* ws = nullptr;
  if (skv::scratch_of_current_device(&ws) != hipSuccess) return SKV_ERR_HIP;
  // The kernels write every word of the scratch they later read (projected queries, one partial result per
  // range, empty ranges included), so nothing needs clearing between calls.
  return skv_decode_attention(layer, q, out, n_ctx, scale, ws, (size_t)SKV_STATIC_SCRATCH_BYTES, stream);
}
