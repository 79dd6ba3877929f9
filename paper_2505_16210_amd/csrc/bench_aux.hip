// libnqkv_benchaux: measurement helpers for the benchmark, built as a library of their own so
// that the product library exports the method and nothing else.
//   nqkv_aux_read_stream  a plain 128-bit read stream over a buffer: what the memory system of the
//                         box delivers to the simplest possible reader, quoted next to the
//                         published peak.  The loads carry the non-temporal hint, as the kernels'
//                         own streaming loads do (measured 7.1 TB/s with it, 6.2 without).
//   nqkv_aux_copy         a plain copy kernel of known size: the yardstick that HBM byte counters
//                         are scaled by.
//   nqkv_aux_empty_launch a kernel that does nothing: the cost of one launch (one graph node).
//   nqkv_aux_mix_stream   a plain kernel that reads R and writes W bytes in a fixed ratio: what the
//                         memory system delivers to the simplest kernel with the read : write mix
//                         of the quantizer (about 4 : 1) or of the dequantizer (1 : 4).  A mixed
//                         stream runs well below a pure read stream on this chip, so this, not
//                         the read stream, is the yardstick for those two kernels.
#include "../../include/nqkv_benchaux.h"

#include <hip/hip_runtime.h>
#include <stdint.h>

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

__global__ __launch_bounds__(256) void copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, uint64_t n_vec) {
  const uint64_t stride = (uint64_t)gridDim.x * 256;
  for (uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x; i < n_vec; i += stride) dst[i] = src[i];
}

__global__ void empty_kernel() {}

// One workgroup per tile: READS 4 KiB pieces in (one 16-byte load per lane each, all issued before
// any is used), WRITES 4 KiB pieces out, all contiguous, all with the non-temporal hint.  What is
// written is a cheap function of what was read, so neither side can be optimised away.
template <int READS, int WRITES>
__global__ __launch_bounds__(256) void mix_stream_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst) {
  const u32x4* s = src + (uint64_t)blockIdx.x * (256 * READS) + threadIdx.x;
  u32x4 v[READS];
#pragma unroll
  for (int r = 0; r < READS; ++r) v[r] = __builtin_nontemporal_load(s + r * 256);
  u32x4 o = v[0];
#pragma unroll
  for (int r = 1; r < READS; ++r) o ^= v[r];
  u32x4* d = dst + (uint64_t)blockIdx.x * (256 * WRITES) + threadIdx.x;
#pragma unroll
  for (int w = 0; w < WRITES; ++w) __builtin_nontemporal_store(o + (unsigned)w, d + w * 256);
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace
}  // namespace nqkv

extern "C" {

int nqkv_aux_read_stream(const void* src, size_t bytes, void* checksums, void* hip_stream) {
  using namespace nqkv;
  if (!src || !checksums || !aligned16(src) || !aligned16(checksums) || (bytes % 16) != 0) return -1;
  hipLaunchKernelGGL(read_stream_kernel, dim3(NQKV_AUX_PROBE_WORKGROUPS), dim3(kProbeThreads), 0,
                     static_cast<hipStream_t>(hip_stream), static_cast<const uint4*>(src), (uint64_t)(bytes / 16),
                     static_cast<uint32_t*>(checksums));
  return hipGetLastError() == hipSuccess ? 0 : -4;
}

int nqkv_aux_copy(void* dst, const void* src, size_t bytes, void* hip_stream) {
  using namespace nqkv;
  if (!src || !dst || !aligned16(src) || !aligned16(dst) || (bytes % 16) != 0) return -1;
  if (bytes == 0) return 0;
  hipLaunchKernelGGL(copy_kernel, dim3(8192), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                     static_cast<const uint4*>(src), static_cast<uint4*>(dst), (uint64_t)(bytes / 16));
  return hipGetLastError() == hipSuccess ? 0 : -4;
}

int nqkv_aux_mix_stream(const void* src, size_t src_bytes, void* dst, size_t dst_bytes, int reads, int writes,
                        size_t* tiles_out, void* hip_stream) {
  using namespace nqkv;
  if (!src || !dst || !tiles_out || !aligned16(src) || !aligned16(dst)) return -1;
  if (!((reads == 4 && writes == 1) || (reads == 1 && writes == 4) || (reads == 1 && writes == 1))) return -1;
  // whole tiles only, as many as both buffers hold: every access stays inside them
  size_t tiles = src_bytes / (4096u * (size_t)reads);
  if (dst_bytes / (4096u * (size_t)writes) < tiles) tiles = dst_bytes / (4096u * (size_t)writes);
  if (tiles > 0x7fffffffu) tiles = 0x7fffffffu;
  *tiles_out = tiles;
  if (tiles == 0) return 0;
  const dim3 grid((unsigned)tiles), block(256);
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const u32x4* s = static_cast<const u32x4*>(src);
  u32x4* d = static_cast<u32x4*>(dst);
  if (reads == 4) hipLaunchKernelGGL((mix_stream_kernel<4, 1>), grid, block, 0, stream, s, d);
  else if (writes == 4) hipLaunchKernelGGL((mix_stream_kernel<1, 4>), grid, block, 0, stream, s, d);
  else hipLaunchKernelGGL((mix_stream_kernel<1, 1>), grid, block, 0, stream, s, d);
  return hipGetLastError() == hipSuccess ? 0 : -4;
}

int nqkv_aux_empty_launch(void* hip_stream) {
  hipLaunchKernelGGL(nqkv::empty_kernel, dim3(1), dim3(64), 0, static_cast<hipStream_t>(hip_stream));
  return hipGetLastError() == hipSuccess ? 0 : -4;
}

}  // extern "C"
