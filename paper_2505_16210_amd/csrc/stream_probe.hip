// Measurement helper, not part of the method: a plain 128-bit read stream over a buffer, so
// that a benchmark can quote the kernels' bandwidth against what the memory system of the box
// delivers to the simplest possible reader, next to the published peak.  The loads carry the
// non-temporal hint, as the kernels' own streaming loads do: measured 7.1 TB/s with it, 6.2 without.
#include "nqkv_internal.h"

namespace nqkv {
namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
constexpr int kProbeThreads = 256;
constexpr int kProbeUnroll = 4;          // 16-byte loads in flight per lane

// Grid-stride over 16-byte vectors: consecutive workgroups read consecutive 16 KiB tiles.
// Every word read is folded (xor) into one checksum per workgroup, which keeps the loads alive
// and lets a test verify that the whole buffer was read exactly once.
__global__ __launch_bounds__(kProbeThreads) void read_stream_kernel(const uint4* __restrict__ src, uint64_t n_vec,
                                                                    uint32_t* __restrict__ checksums) {
  __shared__ uint32_t red[kProbeThreads];
  uint32_t acc = 0;
  const uint64_t stride = (uint64_t)gridDim.x * kProbeThreads * kProbeUnroll;
  for (uint64_t i = (uint64_t)blockIdx.x * kProbeThreads * kProbeUnroll + threadIdx.x; i < n_vec; i += stride) {
    uint4 v[kProbeUnroll];
#pragma unroll
    for (int u = 0; u < kProbeUnroll; ++u) {
      const uint64_t j = i + (uint64_t)u * kProbeThreads;
      if (j < n_vec) {
        const u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src) + j);
        v[u] = make_uint4(t.x, t.y, t.z, t.w);
      } else {
        v[u] = make_uint4(0, 0, 0, 0);
      }
    }
#pragma unroll
    for (int u = 0; u < kProbeUnroll; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int s = kProbeThreads / 2; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) red[threadIdx.x] ^= red[threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0) checksums[blockIdx.x] = red[0];
}

}  // namespace

hipError_t launch_read_stream(const void* src, uint64_t bytes, uint32_t* checksums, int workgroups, hipStream_t stream) {
  hipLaunchKernelGGL(read_stream_kernel, dim3((unsigned)workgroups), dim3(kProbeThreads), 0, stream,
                     static_cast<const uint4*>(src), bytes / 16, checksums);
  return hipGetLastError();
}

}  // namespace nqkv
