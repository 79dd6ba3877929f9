// Library-owned scratch memory for callers that cannot allocate: the split-K workspace of the
// attention kernels as a fixed array in device memory, so that an entry point can run without any
// hipMalloc (under graph capture, in a serving loop, in a harness that forbids allocation).
//
// Every GPU the library runs on holds its own copy of the array, at its own address, from the
// moment the code object is loaded there until the process ends.  The array's name is only a
// host-side stand-in in host code: the device address of the current device's copy is looked up
// once per device with hipGetSymbolAddress and that pointer is what kernels and fills receive.
#include "nqkv_internal.h"

#include <mutex>

namespace nqkv {
namespace {

static __device__ __align__(256) __attribute__((used)) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_lookup_mutex;
void* g_scratch_of_device[kMaxDevices];      // device address of `scratch` on device i, once looked up

// Sets n 32-bit words to zero.  A kernel, not hipMemsetAsync: memset nodes recorded into a HIP
// graph have produced wrong results on replay on this platform.
__global__ __launch_bounds__(256) void clear_words_kernel(uint32_t* __restrict__ p, int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0u;
}

}  // namespace

hipError_t static_scratch(void** ptr_out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> hold(g_lookup_mutex);
  if (!g_scratch_of_device[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!ptr) return hipErrorInvalidSymbol;
    g_scratch_of_device[dev] = ptr;
  }
  *ptr_out = g_scratch_of_device[dev];
  return hipSuccess;
}

hipError_t launch_clear_words(uint32_t* words, int n, hipStream_t stream) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(clear_words_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, words, n);
  return hipGetLastError();
}

}  // namespace nqkv
