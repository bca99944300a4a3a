// Scratch memory of arrow_spmm_static: one array per GPU the library is loaded on, part of the
// library's code object and held until the process ends.  In host code the array's name is only a
// stand-in for the symbol; the device address is looked up once per device (with that device
// current) and that pointer is what the kernels get.
#include <hip/hip_runtime.h>

#include <mutex>
#include <string>

#include "arrow.h"
#include "arrow_internal.h"

namespace {

static __device__ __align__(256) unsigned char scratch[ARROW_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
unsigned char* g_scratch_ptr[kMaxDevices] = {};

}  // namespace

namespace arrow {

// device address of the current device's scratch array (NULL + a description on failure)
unsigned char* static_scratch(std::string& err) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    err = std::string("static scratch: no usable current device: ") + hipGetErrorString(e);
    return nullptr;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) {
      err = std::string("static scratch: hipGetSymbolAddress failed: ") + hipGetErrorString(e);
      return nullptr;
    }
    g_scratch_ptr[dev] = static_cast<unsigned char*>(ptr);
  }
  return g_scratch_ptr[dev];
}

}  // namespace arrow
