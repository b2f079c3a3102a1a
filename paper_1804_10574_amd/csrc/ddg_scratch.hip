// Static device scratch for the entry point that must not allocate (ddg_forward_eval_static):
// one array per GPU, part of the library's code object, held until the process ends.
//
// The array's name is a host-side stand-in in host code, not a device address. Its device
// address is looked up once per device with hipGetSymbolAddress (with that device current);
// all host code uses the looked-up pointer (kernel arguments, copies), never the name.
#include <hip/hip_runtime.h>

#include <mutex>

#include "ddg_kernels.h"

static __device__ __align__(256) unsigned char scratch[DDG_STATIC_SCRATCH_BYTES];

namespace ddg {

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_mu;
void* g_ptr[kMaxDevices] = {nullptr};   // device address of `scratch` on each GPU, once looked up
}  // namespace

hipError_t static_scratch(void** ptr, size_t* bytes) {
  *ptr = nullptr;
  *bytes = 0;
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_mu);
  if (!g_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_ptr[dev] = p;
  }
  *ptr = g_ptr[dev];
  *bytes = DDG_STATIC_SCRATCH_BYTES;
  return hipSuccess;
}

}  // namespace ddg
