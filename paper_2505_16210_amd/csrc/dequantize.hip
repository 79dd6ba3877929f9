// Packed cache -> fp16 (paper Fig. 5 caption and Sec. 3.2: X' = dequantize(I); the index is
// looked up in the table and restored to FP16).  out = fp16_rne(fl32(level[code] * scale)).
// gfx950 only.  The kernel writes four times the bytes it reads, so the mapping follows the
// stores: one lane owns 8 consecutive elements of a token row -- k bytes of codes in, one 16-byte
// store out -- and consecutive lanes own consecutive chunks, so a store instruction of a wave
// covers 1 KiB of whole rows (contiguous when the rows are) and a code load 64 k bytes.  A
// workgroup walks over kPasses row groups with all of their loads issued before the first use.
#include "decode_common.h"
#include "nqkv_internal.h"

namespace nqkv {
namespace {

// lanes per workgroup: 128 at 4 bits, 256 at 2 and 3 (measured: 4 % faster each than the other way round)
template <int KBITS> constexpr int kThreadsFor = (KBITS == 4) ? 128 : 256;
constexpr int kPasses = 4;
constexpr uint32_t kDropStore = 0xffffffffu;      // an offset outside every buffer: the store is dropped
constexpr int kNonTemporal = 2;                   // cache-policy bit of a buffer instruction: read or written once
constexpr int64_t kCacheableOutputBytes = 64ll << 20;   // a quarter of the 256 MB last-level cache

// NT: the stores carry the non-temporal hint (output too large for the last-level cache to keep
// for its reader: measured 3-5 % faster at 0.5-7 GB, while a 64 MiB output is better left cacheable).
template <int KBITS, int D, int BLK, bool NT>
__global__ __launch_bounds__(kThreadsFor<KBITS>) void dequantize_kernel(const QuantParams p) {
  constexpr int kThreads = kThreadsFor<KBITS>;
  constexpr uint32_t CPR = D / 8;              // 8-element chunks per row
  constexpr uint32_t RPP = kThreads / CPR;     // rows per pass of the workgroup
  constexpr uint32_t NB = D / BLK;
  constexpr uint32_t kRowBytes = D * KBITS / 8, kScaleRowBytes = NB * 2;
  constexpr uint32_t kMask = (1u << KBITS) - 1u;
  __shared__ float lv[1 << KBITS];
  // The level table (2^k floats in LDS), filled by the first 2^k threads.  Where it is filled
  // matters by a few per cent and was settled by measurement (B16 H56 D128 S16384, one tensor):
  //   k = 4: after the code loads have been issued, from scalar registers   758-778 us
  //          (before them, by a load indexed with the thread: 778-789; before them, from
  //          scalar registers: 797)
  //   k = 3: before the loads, by a load indexed with the thread            780 us
  //          (after them: 800-805; before them from scalar registers: 814)
  //   k = 2: 704-712 us every way
  // A thread-indexed read of the kernel-argument array is a vector load with a barrier behind it;
  // in front of the code loads it delays each workgroup's start a little, which at k = 3 -- twice
  // the code loads in flight -- spreads the workgroups' phases apart and helps; behind the code
  // loads it would queue after them (the memory counter is positional), hence the scalar form there.
  if constexpr (KBITS == 3) {
    if (threadIdx.x < (1 << KBITS)) lv[threadIdx.x] = p.levels.v[threadIdx.x];
    __syncthreads();
  }

  const uint32_t b = blockIdx.z, h = blockIdx.y;
  const int64_t row0 = ((int64_t)b * p.H + h) * p.cap_tokens + p.tok_off;
  const uint32_t n = (uint32_t)p.n_tokens;
  // Descriptors of this (batch, head) slab: rows past n_tokens read zeros and their stores are
  // dropped, so every pass issues the same unconditional instructions.  (The host has checked
  // that all three byte ranges fit 31 bits.)
  const __amdgpu_buffer_rsrc_t code_r = __builtin_amdgcn_make_buffer_rsrc(
      p.t[0].codes + row0 * kRowBytes, 0, (int)(n * kRowBytes), kBufferFlags);
  const __amdgpu_buffer_rsrc_t scale_r = __builtin_amdgcn_make_buffer_rsrc(
      p.t[0].scales + row0 * NB, 0, (int)(n * kScaleRowBytes), kBufferFlags);
  const uint32_t st = (uint32_t)p.stride_t;
  const __amdgpu_buffer_rsrc_t dst_r = __builtin_amdgcn_make_buffer_rsrc(
      p.t[0].dst + (int64_t)b * p.stride_b + (int64_t)h * p.stride_h, 0, (int)(((n - 1u) * st + D) * 2u), kBufferFlags);

  const uint32_t r = threadIdx.x / CPR, c = threadIdx.x % CPR;
  const uint32_t t0 = blockIdx.x * (kPasses * RPP) + r;

  uint32_t w[kPasses];
  uint16_t sc[kPasses];
#pragma unroll
  for (int u = 0; u < kPasses; ++u) {
    const uint32_t t = t0 + u * RPP;
    const uint32_t off = t * kRowBytes + c * KBITS;
    if constexpr (KBITS == 4) {
      w[u] = __builtin_amdgcn_raw_buffer_load_b32(code_r, off, 0, kNonTemporal);
    } else if constexpr (KBITS == 2) {
      w[u] = __builtin_amdgcn_raw_buffer_load_b16(code_r, off, 0, kNonTemporal);
    } else {
      // 3 bytes at any byte offset: the two aligned dwords around them (each range-checked on
      // its own), shifted down by the offset's low bits
      const uint32_t a = off & ~3u;
      const uint32_t lo = __builtin_amdgcn_raw_buffer_load_b32(code_r, a, 0, 0);
      const uint32_t hi = __builtin_amdgcn_raw_buffer_load_b32(code_r, a + 4u, 0, 0);
      w[u] = __builtin_amdgcn_alignbyte(hi, lo, off & 3u);
    }
    sc[u] = __builtin_amdgcn_raw_buffer_load_b16(scale_r, t * kScaleRowBytes + ((c * 8u) / BLK) * 2u, 0, 0);
  }

  if constexpr (KBITS != 3) {
    float mine = 0.0f;
#pragma unroll
    for (int i = 0; i < (1 << KBITS); ++i) {
      float level_i = p.levels.v[i];
      asm volatile("" : "+s"(level_i));        // a value in a scalar register, not an address to select
      mine = (threadIdx.x == (unsigned)i) ? level_i : mine;
    }
    if (threadIdx.x < (1 << KBITS)) lv[threadIdx.x] = mine;
    __syncthreads();
  }

#pragma unroll
  for (int u = 0; u < kPasses; ++u) {
    const uint32_t t = t0 + u * RPP;
    const float s32 = (float)__builtin_bit_cast(_Float16, sc[u]);
    uint32_t o[4];
#pragma unroll
    for (int e = 0; e < 8; e += 2) {
      float lo = lv[(w[u] >> (KBITS * e)) & kMask] * s32;                // one fp32 rounding
      float hi = lv[(w[u] >> (KBITS * (e + 1))) & kMask] * s32;
      // Keep the fp32 product as its own instruction: without this the compiler merges the
      // multiply and the conversion into one mixed-precision fma with a +0 addend, which rounds
      // once instead of twice and turns -0 products into +0.
      asm volatile("" : "+v"(lo), "+v"(hi));
      const uint32_t l16 = __builtin_bit_cast(unsigned short, (_Float16)lo);  // round to nearest even
      const uint32_t h16 = __builtin_bit_cast(unsigned short, (_Float16)hi);
      o[e >> 1] = l16 | (h16 << 16);
    }
    const u32x4_t v = {o[0], o[1], o[2], o[3]};
    // (the row test rather than the range check alone: t * stride may wrap for rows past the end)
    __builtin_amdgcn_raw_buffer_store_b128(v, dst_r, t < n ? (t * st + c * 8u) * 2u : kDropStore, 0, NT ? kNonTemporal : 0);
  }
}

template <int KBITS, int D, int BLK>
hipError_t launch_one(const QuantParams& p, hipStream_t stream) {
  constexpr int kThreads = kThreadsFor<KBITS>;
  constexpr int64_t kTileRows = kPasses * (kThreads / (D / 8));
  dim3 grid((unsigned)((p.n_tokens + kTileRows - 1) / kTileRows), (unsigned)p.H, (unsigned)p.B);
  const int64_t out_bytes = (int64_t)p.B * p.H * p.n_tokens * D * 2;
  if (out_bytes > kCacheableOutputBytes)
    hipLaunchKernelGGL((dequantize_kernel<KBITS, D, BLK, true>), grid, dim3(kThreads), 0, stream, p);
  else
    hipLaunchKernelGGL((dequantize_kernel<KBITS, D, BLK, false>), grid, dim3(kThreads), 0, stream, p);
  return hipGetLastError();
}

template <int KBITS>
hipError_t launch_k(const QuantParams& p, int D, int blk, hipStream_t stream) {
  if (D == 64 && blk == 64) return launch_one<KBITS, 64, 64>(p, stream);
  if (D == 128 && blk == 64) return launch_one<KBITS, 128, 64>(p, stream);
  if (D == 128 && blk == 128) return launch_one<KBITS, 128, 128>(p, stream);
  return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_dequantize(const QuantParams& p, int D, int k, int blk, hipStream_t stream) {
  switch (k) {
    case 2: return launch_k<2>(p, D, blk, stream);
    case 3: return launch_k<3>(p, D, blk, stream);
    case 4: return launch_k<4>(p, D, blk, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace nqkv
