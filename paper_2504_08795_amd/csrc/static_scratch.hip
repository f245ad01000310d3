// Device memory that exists without any allocation call: a file-scope array in the library's own device image.
//
// daris_forward_static (daris.h) serves callers that must not allocate device memory.  The activation tensors and the
// split-K partial sums of the network it runs live in this array instead of in buffers obtained with hipMalloc.  Each
// GPU the library runs on holds its own copy of the array, at its own address, from the first daris_init on that GPU
// until the process ends.
//
// In host code the array's name is only a handle for the HIP runtime, not a device address: the address is looked up
// once per device with hipGetSymbolAddress (below) and only that pointer is ever handed to kernels or copies.
#include <hip/hip_runtime.h>

#include <string>

#include "static_scratch.h"

static __device__ __align__(256) unsigned char scratch[DARIS_STATIC_SCRATCH_BYTES];

namespace daris {

namespace {
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {nullptr};  // per HIP device: where that GPU's copy of `scratch` lies
}  // namespace

std::string static_scratch_init(int device) {
  if (device < 0 || device >= kMaxDevices) return "device index " + std::to_string(device) + " out of range for the static scratch";
  if (g_scratch_ptr[device]) return "";
  int cur = -1;
  hipError_t e = hipGetDevice(&cur);
  if (e != hipSuccess) return std::string("hipGetDevice: ") + hipGetErrorString(e);
  if (cur != device) return "static scratch set-up needs device " + std::to_string(device) + " current, but device " + std::to_string(cur) + " is";
  void* ptr = nullptr;
  e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
  if (e != hipSuccess || !ptr) return std::string("hipGetSymbolAddress(scratch): ") + (e != hipSuccess ? hipGetErrorString(e) : "null address");
  if (reinterpret_cast<uintptr_t>(ptr) % 256 != 0) return "the static scratch is not 256-byte aligned";
  g_scratch_ptr[device] = ptr;
  return "";
}

void* static_scratch_ptr(int device) { return (device >= 0 && device < kMaxDevices) ? g_scratch_ptr[device] : nullptr; }

}  // namespace daris
