// Pieces shared by the attention kernels over the packed cache: the byte-indexed look-up table
// in LDS that turns codes into fp16 levels, raw buffer loads of code rows, wave reductions and the
// write-through stores used for split results.  Device code only.
#pragma once

#include "nqkv_internal.h"

namespace nqkv {
namespace {

constexpr int kLutWords = 16384;         // 64 KiB: 256 rows of 256 bytes (k = 4, 2); k = 3 uses 2048
// Running maximum of a wave that has seen no token yet: a finite number below every real score
// instead of -inf, so that an item without any token (a split beyond the end of a short
// sequence) comes out as (m, l = 0, o = 0) -- exp2(m - m) = 1 times zero sums -- where -inf
// would make exp2(-inf - -inf) = NaN.  Real scores lift the maximum on their first trip and
// exp2(kNoScore - score) is exactly 0.
constexpr float kNoScore = -1.0e30f;

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
constexpr int kQuadXor1 = 0xB1, kQuadXor2 = 0x4E, kRowHalfMirror = 0x141, kRowMirror = 0x140;

// SAME: lanes that already hold equal values -- 1, 2 or 4 neighbours (an aligned pair, a quad)
template <int SAME = 1>
__device__ __forceinline__ float wave_max(float v) {
  if (SAME < 2) v = fmaxf(v, dpp_f<kQuadXor1>(v));
  if (SAME < 4) v = fmaxf(v, dpp_f<kQuadXor2>(v));
  v = fmaxf(v, dpp_f<kRowHalfMirror>(v));
  v = fmaxf(v, dpp_f<kRowMirror>(v));
  const int i = __builtin_bit_cast(int, v);
  const float a = __builtin_bit_cast(float, __builtin_amdgcn_readlane(i, 0));
  const float b = __builtin_bit_cast(float, __builtin_amdgcn_readlane(i, 16));
  const float c = __builtin_bit_cast(float, __builtin_amdgcn_readlane(i, 32));
  const float d = __builtin_bit_cast(float, __builtin_amdgcn_readlane(i, 48));
  return fmaxf(fmaxf(a, b), fmaxf(c, d));
}

__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_f<kQuadXor1>(v);
  v += dpp_f<kQuadXor2>(v);
  v += dpp_f<kRowHalfMirror>(v);
  v += dpp_f<kRowMirror>(v);
  const int i = __builtin_bit_cast(int, v);
  const float a = __builtin_bit_cast(float, __builtin_amdgcn_readlane(i, 0));
  const float b = __builtin_bit_cast(float, __builtin_amdgcn_readlane(i, 16));
  const float c = __builtin_bit_cast(float, __builtin_amdgcn_readlane(i, 32));
  const float d = __builtin_bit_cast(float, __builtin_amdgcn_readlane(i, 48));
  return (a + b) + (c + d);
}

// bits [pos, pos+n) of a little-endian dword array; pos, n compile-time after unrolling
template <int NDW>
__device__ __forceinline__ uint32_t field(const uint32_t (&w)[NDW], int pos, int n) {
  const int i = pos >> 5, sh = pos & 31;
  uint32_t v = w[i] >> sh;
  if (sh + n > 32 && i + 1 < NDW) v |= w[i + 1] << (32 - sh);
  return v & ((1u << n) - 1u);
}

// ------------------------------------------------------------------ look-up tables in LDS
// k = 4: row = byte (2 codes), 256 B: 64 copies of dword {fp16 level[lo nibble], level[hi nibble]}
// k = 2: row = byte (4 codes), 256 B: 32 copies of 2 dwords {l[c0], l[c1]}, {l[c2], l[c3]}
// k = 3: row = 6 bits (2 codes), 128 B: 32 copies of dword {level[lo 3 bits], level[hi 3 bits]}
// Lane L reads copy L (k = 4), L & 31 (k = 2, 3).
//
// Built from the 16 fp16 levels in the kernel arguments: every index that depends only on the
// loop counter is a compile-time constant (a scalar register), the per-thread ones are picked
// once with a short select chain -- no LDS reads, one barrier.
template <class Params>
__device__ __forceinline__ uint32_t pick_level(const Params& p, uint32_t idx, int n) {
  uint32_t v = 0;
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    if (j < n) v = (idx == (uint32_t)j) ? (uint32_t)p.lut_levels[j] : v;
  }
  return v;
}

template <int KBITS, class Params>
__device__ __forceinline__ void build_lut(const Params& p, uint32_t* smem) {
  if constexpr (KBITS == 4) {
    // word index = e * 64 + copy; thread t writes entries e = (t >> 6) + 8 i, copy = t & 63:
    // low nibble (t >> 6) + 8 (i & 1), high nibble i >> 1
    const uint32_t copy = threadIdx.x & 63, e0 = threadIdx.x >> 6;       // e0 in [0, 8)
    const uint32_t lo_even = pick_level(p, e0, 16), lo_odd = pick_level(p, e0 + 8, 16);
#pragma unroll
    for (int i = 0; i < 32; ++i) {
      const uint32_t hi = p.lut_levels[i >> 1];
      smem[(e0 + 8 * i) * 64 + copy] = ((i & 1) ? lo_odd : lo_even) | (hi << 16);
    }
  } else if constexpr (KBITS == 3) {
    // word index = e * 32 + copy; thread t: e = (t >> 5) + 16 i (6 bits), copy = t & 31:
    // low code (t >> 5) & 7, high code (t >> 8) + 2 i
    const uint32_t copy = threadIdx.x & 31, e0 = threadIdx.x >> 5;       // e0 in [0, 16)
    const uint32_t lo = pick_level(p, e0 & 7, 8);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t hi_a = p.lut_levels[2 * i], hi_b = p.lut_levels[2 * i + 1];
      smem[(e0 + 16 * i) * 32 + copy] = lo | (((e0 >> 3) ? hi_b : hi_a) << 16);
    }
  } else {
    // word index = e * 64 + c; thread t: e = (t >> 6) + 8 i, c = t & 63 (dword of the row: even
    // dwords hold {c0, c1}, odd dwords {c2, c3});
    // c0 = e0 & 3, c1 = (e0 >> 2) + 2 (i & 1), c2 = (i >> 1) & 3, c3 = i >> 3
    const uint32_t c = threadIdx.x & 63, e0 = threadIdx.x >> 6;          // e0 in [0, 8)
    const uint32_t c0 = pick_level(p, e0 & 3, 4);
    const uint32_t c1_even = pick_level(p, e0 >> 2, 4), c1_odd = pick_level(p, (e0 >> 2) + 2, 4);
#pragma unroll
    for (int i = 0; i < 32; ++i) {
      const uint32_t lo = c0 | (((i & 1) ? c1_odd : c1_even) << 16);
      const uint32_t hi = (uint32_t)p.lut_levels[(i >> 1) & 3] | ((uint32_t)p.lut_levels[i >> 3] << 16);
      smem[(e0 + 8 * i) * 64 + c] = (c & 1) ? hi : lo;
    }
  }
  __syncthreads();
}

// LDS byte address of the table row selected by byte B (0..3) of code dword w, this lane's
// copy:  v_perm_b32 -> byte0 = lane_off byte0, byte1 = w byte B, bytes 2 and 3 = 0.
template <int B>
__device__ __forceinline__ uint32_t row_addr(uint32_t w, uint32_t lane_off) {
  return __builtin_amdgcn_perm(w, lane_off, 0x0c0c0000u | ((4u + B) << 8));
}

// ------------------------------------------------------------------ HBM loads
// All cache reads are raw buffer loads: a scalar descriptor per item (base = first token of the
// item's range, num_records = bytes of the range), one per-lane byte offset in a VGPR, and the
// four round offsets of a trip as instruction immediates.  That keeps 64-bit addresses out of
// the vector ALU and out of vector registers.  Only voffset (not a scalar offset) takes part in
// the hardware range check, so the trip's offset is added into voffset: lanes past the end of
// the range then read zeros -- code 0, scale 0 -- and never touch memory outside the range.
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x3_t __attribute__((ext_vector_type(3)));
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
constexpr int kBufferFlags = 0x00020000;   // raw buffer, 32-bit data format (gfx9 family)
// Cache-policy bits of a buffer instruction (its last argument): bit 1 is the non-temporal hint.
// A stream that is read once and consumed a whole cache line per instruction runs faster with it
// (a plain 128-bit read stream: 7.1 against 6.2 TB/s on this chip).  Loads that take a line in
// pieces, several instructions apart, must not carry it: the line is gone by the second piece.
constexpr int kStreamOnce = 2;

template <int KBITS>
__device__ __forceinline__ void load_codes(__amdgpu_buffer_rsrc_t rsrc, uint32_t voff, uint32_t soff,
                                           uint32_t (&w)[KBITS]) {
  if constexpr (KBITS == 4) {
    const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, voff, soff, kStreamOnce);
    w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
  } else if constexpr (KBITS == 3) {
    const u32x3_t v = __builtin_amdgcn_raw_buffer_load_b96(rsrc, voff, soff, kStreamOnce);
    w[0] = v.x; w[1] = v.y; w[2] = v.z;
  } else {
    const u32x2_t v = __builtin_amdgcn_raw_buffer_load_b64(rsrc, voff, soff, kStreamOnce);
    w[0] = v.x; w[1] = v.y;
  }
}

// Device-wide visible 32-bit store / load of a float (write-through / cache-bypassing).
__device__ __forceinline__ void store_agent(uint32_t* p, float v) {
  __hip_atomic_store(p, __builtin_bit_cast(uint32_t, v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float load_agent(const uint32_t* p) {
  return __builtin_bit_cast(float, __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
}

}  // namespace
}  // namespace nqkv
