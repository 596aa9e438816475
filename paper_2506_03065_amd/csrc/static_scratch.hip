// A file-scope buffer in device memory.  Its name is a host-side stand-in, not a
// device address: host code must resolve it with hipGetSymbolAddress, once per
// device with that device current, and pass the resolved pointer to kernels,
// copies and fills.
#include "static_scratch.h"

#include <mutex>

namespace svd {
namespace {

static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_mu;
void* g_ptr[kMaxDevices] = {};

}  // namespace

hipError_t static_scratch(void** ptr, size_t* bytes) {
  if (!ptr || !bytes) return hipErrorInvalidValue;
  int dev = 0;
  if (hipError_t e = hipGetDevice(&dev); e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_mu);
  if (!g_ptr[dev]) {
    void* p = nullptr;
    if (hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)); e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_ptr[dev] = p;
  }
  *ptr = g_ptr[dev];
  *bytes = kStaticScratchBytes;
  return hipSuccess;
}

}  // namespace svd
