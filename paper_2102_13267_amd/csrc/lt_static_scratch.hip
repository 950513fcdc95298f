// The library's own device scratch, for callers that cannot allocate device memory (code under
// HIP graph capture, serving loops, harnesses that forbid hipMalloc): lt_barrier_static runs a plan
// with its reduction scratch and its temporaries here instead of in a caller-supplied workspace.
//
// One array per GPU, held from the moment the library's code is loaded on that GPU until the
// process ends.  `scratch` below is a host-side stand-in for the device symbol, not an address:
// host code gets the array's address on a device from hipGetSymbolAddress, once per device with
// that device current, and uses that pointer from then on (kernel arguments, fills).
#include <hip/hip_runtime.h>

#include <mutex>

#include "lt_launch.h"

namespace ltk {

static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_lock;
void* g_ptr[kMaxDevices] = {};
}  // namespace

// Address of the static scratch on `device` (which must be the current device).
hipError_t static_scratch(int device, void** ptr, size_t* bytes) {
  if (device < 0 || device >= kMaxDevices || !ptr || !bytes) return hipErrorInvalidValue;
  std::lock_guard<std::mutex> guard(g_lock);
  if (!g_ptr[device]) {
    int current = -1;
    hipError_t e = hipGetDevice(&current);
    if (e != hipSuccess) return e;
    if (current != device) return hipErrorInvalidDevice;
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_ptr[device] = p;
  }
  *ptr = g_ptr[device];
  *bytes = kStaticScratchBytes;
  return hipSuccess;
}

__global__ void lt_fill_u32_kernel(uint32_t* p, uint32_t n, uint32_t value) {
  const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = value;
}

// p[0 .. n) = value, as a kernel (a memset node inside a captured graph is not an option here).
hipError_t launch_fill_u32(uint32_t* p, uint32_t n, uint32_t value, hipStream_t s) {
  if (!p) return hipErrorInvalidValue;
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(lt_fill_u32_kernel, dim3((n + 255u) / 256u), dim3(256), 0, s, p, n, value);
  return hipGetLastError();
}

}  // namespace ltk
