// A fixed block of device memory inside the library's code object, for the one entry
// point that may not allocate (gco_round_repair_static).  Every GPU the library runs on
// holds its own copy of the array, at its own address, until the process ends.
#include <hip/hip_runtime.h>

#include <mutex>

#include "gco_internal.h"

namespace gco {

namespace {

static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_lock;
void* g_ptr[kMaxDevices] = {};  // device address of `scratch` on device d, once looked up

}  // namespace

// Device address of the static scratch block on the CURRENT device (looked up once per
// device with that device current; in host code the array's name is only a handle for
// this lookup, never an address).  Returns hipSuccess and the pointer, or the error.
hipError_t static_scratch_for_current_device(void** out) {
  *out = nullptr;
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> guard(g_lock);
  if (g_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    g_ptr[dev] = ptr;
  }
  *out = g_ptr[dev];
  return hipSuccess;
}

}  // namespace gco
