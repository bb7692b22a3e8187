// Library-owned scratch memory for callers that cannot allocate (code under HIP graph capture,
// serving loops that hold no workspace, harnesses that forbid hipMalloc): a fixed array in
// device memory that every GPU the library runs on holds until the process ends.
#include <hip/hip_runtime.h>

#include <mutex>
#include <string>

#include "rosaq_internal.h"

namespace rosaq {

// Rotated activations, tickets and fp32 partial tiles of one call, laid out exactly like a
// caller's workspace.  In host code this name only stands for the symbol: the address the
// kernels get comes from hipGetSymbolAddress below, once per device.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

int static_scratch(void** ptr_out) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void* ptrs[kMaxDevices] = {};
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) {
    set_error(std::string("hipGetDevice: ") + hipGetErrorString(e));
    return ROSAQ_ERR_HIP;
  }
  if (dev < 0 || dev >= kMaxDevices) {
    set_error("device ordinal beyond the static scratch table");
    return ROSAQ_ERR_HIP;
  }
  std::lock_guard<std::mutex> lock(mu);
  if (ptrs[dev] == nullptr) {
    void* p = nullptr;   // each device holds its own copy of the array at its own address
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || p == nullptr) {
      set_error(std::string("hipGetSymbolAddress(scratch): ") + hipGetErrorString(e));
      return ROSAQ_ERR_HIP;
    }
    ptrs[dev] = p;
  }
  *ptr_out = ptrs[dev];
  return ROSAQ_OK;
}

}  // namespace rosaq
