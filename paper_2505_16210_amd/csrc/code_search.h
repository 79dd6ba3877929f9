// Device-side code search shared by the quantizer kernels and the fused decode step:
// code(x) = #{ j : x > fl32(t_j * s) } for the eight fp16 values of one 16-byte chunk.
// See quantize.hip for the derivation of the cell-table path.
#pragma once

#include "nqkv_internal.h"

namespace nqkv {
namespace code_search {

// (the cell grid's constants -- kCells, kCellScale, kCellBias, kCellMargin -- are shared with the
// host, which builds the table: see nqkv_internal.h)
// Adding 2^20 puts the integer part of u in mantissa bits [3, 10): (bits & 0x3f8) is then
// the byte offset of an 8-byte table entry.
constexpr float kCellMagic = 1048576.0f + kCellBias;

typedef unsigned short us2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t pk_max_u16(uint32_t a, uint32_t b) {
  return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(us2, a),
                                                                __builtin_bit_cast(us2, b)));
}

template <int CTRL>
__device__ __forceinline__ uint32_t dpp(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, true);
}
// DPP controls: lane permutes inside a row of 16 lanes.
constexpr int kQuadXor1 = 0xB1;       // quad_perm [1,0,3,2]
constexpr int kQuadXor2 = 0x4E;       // quad_perm [2,3,0,1]
constexpr int kRowHalfMirror = 0x141; // lane i <-> 7-i within 8
constexpr int kRowMirror = 0x140;     // lane i <-> 15-i within 16
constexpr int kQuadNext = 0xF9;       // quad_perm [1,2,3,3]: value of the next lane in the quad
constexpr int kQuadOdd = 0xF5;        // quad_perm [1,1,3,3]: value of the odd lane of each pair

__device__ __forceinline__ float half_bits_to_float(uint32_t h) {
  return (float)__builtin_bit_cast(_Float16, (unsigned short)h);
}

// The cell table is built on the host (build_cell_table) and arrives in the kernel arguments;
// each workgroup copies it into LDS once: thread i fetches entry i early, stores it later.  The
// caller provides the barrier.
__device__ __forceinline__ uint2 fetch_cell(const uint32_t* thr, const uint32_t* below) {
  return threadIdx.x < kCells ? make_uint2(thr[threadIdx.x], below[threadIdx.x]) : make_uint2(0, 0);
}
__device__ __forceinline__ void put_cell(const uint2& cell, uint2* cells) {
  if (threadIdx.x < kCells) cells[threadIdx.x] = cell;
}

// Codes of the 8 fp16 values in w against scale bits s_bits, packed LSB-first, KBITS each.
template <int KBITS, bool FAST>
__device__ __forceinline__ uint32_t encode_chunk(const uint4& w, uint32_t s_bits, const LevelTable& lv,
                                                 const uint2* cells) {
  const float s32 = half_bits_to_float(s_bits);
  const uint32_t words[4] = {w.x, w.y, w.z, w.w};
  uint32_t packed = 0;
  if (FAST) {
    const float inv = s_bits ? kCellScale * __builtin_amdgcn_rcpf(s32) : 0.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const uint32_t h = (e & 1) ? (words[e >> 1] >> 16) : (words[e >> 1] & 0xffffu);
      const float x = half_bits_to_float(h);
      const float u = __builtin_fmaf(x, inv, kCellMagic);
      const uint32_t off = __float_as_uint(u) & 0x3f8u;
      const uint2 ent = *reinterpret_cast<const uint2*>(reinterpret_cast<const char*>(cells) + off);
      const float T = __uint_as_float(ent.x) * s32;        // fl32(t * s): one rounding
      const uint32_t code = ent.y + ((x > T) ? 1u : 0u);
      packed |= code << (KBITS * e);
    }
  } else {
    float T[(1 << KBITS) - 1];
#pragma unroll
    for (int j = 1; j < (1 << KBITS); ++j) {
      const float t = (lv.v[j - 1] + lv.v[j]) * 0.5f;
      T[j - 1] = t * s32;                                  // fl32(t * s): one rounding
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const uint32_t h = (e & 1) ? (words[e >> 1] >> 16) : (words[e >> 1] & 0xffffu);
      const float x = half_bits_to_float(h);
      uint32_t code = 0;
#pragma unroll
      for (int j = 0; j < (1 << KBITS) - 1; ++j) code += (x > T[j]) ? 1u : 0u;
      packed |= code << (KBITS * e);
    }
  }
  // all-zero block: every scaled threshold is +-0 and 0 > +-0 is false -> code 0
  return s_bits ? packed : 0u;
}

}  // namespace code_search
}  // namespace nqkv
