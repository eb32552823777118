// The fixed device array behind fl_layer_forward_static: the entry point for callers that cannot
// allocate device memory.  One array per GPU, alive from the moment the library's code is loaded on that
// GPU until the process ends; every call on a GPU shares it.
#include <hip/hip_runtime.h>

#include <mutex>

#include "static_scratch.h"

namespace fl {
namespace {

static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// In host code the array's name only stands for the symbol: the address each GPU gave its copy is looked
// up once per device and kept here.
constexpr int kMaxDevices = 64;
void *g_base[kMaxDevices] = {};
std::mutex g_mu;

}  // namespace

hipError_t static_scratch_base(void **base) {
  *base = nullptr;
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_mu);
  if (!g_base[dev]) {
    void *p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));  // the copy of the current device
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_base[dev] = p;
  }
  *base = g_base[dev];
  return hipSuccess;
}

}  // namespace fl
