// Dequantize-fused decode attention over the packed cache (paper Sec. 3.2, decoding phase:
// X_K' = dequantize(I_K), X_V' = dequantize(I_V), A = Softmax(t_Q X_K'^T), t_O = A X_V').
// The paper materialises X' for the whole cache every step; here the table look-up happens in
// registers between the HBM read of the packed codes and the dot products, so a decode step
// moves only the packed bytes.  gfx950 only; no matrix cores (one query row per head).
//
// Mapping.  Eight-wave workgroups, each building the look-up table once and then walking over
// work items (batch*head, split) with the grid as stride; an item's token range is streamed
// once.  The host sizes the grid: at most two workgroups per compute unit (a persistent grid) for
// short items, one workgroup per item for long ones.  A lane owns 32 consecutive head-dim elements
// of a token (4*k bytes of codes, one block scale), so LPT = D/32 adjacent lanes hold one token and
// a wave load covers 64/LPT tokens with one fully coalesced request (1 KiB at k = 4), marked
// non-temporal: the cache is read once.  Four such loads of K and
// four of V are in flight per wave; the first trip's loads are issued before the look-up table
// is built and the next trip's K loads before the current trip's V arithmetic.
//
// Look-up.  Codes become values through an LDS table indexed by a whole byte of codes
// (k = 4: two codes -> two fp16 levels in one dword; k = 2: four codes -> four fp16 in two
// dwords; k = 3: a 6-bit pair -> one dword).  The kernel is bound by VALU issue as much as by
// HBM, so the address of a look-up must cost one instruction: for k = 4 and k = 2 every table
// row is 256 bytes apart (32 copies of the entry, lane L reading copy L mod 32: no bank
// conflicts), which lets a single
// v_perm_b32 assemble  address = code_byte * 256 + lane_offset  from the code dword and a
// per-lane constant.  (k = 3 pairs are not byte aligned: the 96-bit stream of a lane is shifted
// as a whole so that four pairs at a time start on byte boundaries, see for_each_pair_k3.)
//
// Table precision.  The table holds fp16 numbers.  Rounding the levels themselves to fp16 would
// put a systematic relative error of up to 2^-11 on whole classes of elements, which the
// exponential amplifies by the score range; instead the host picks a factor gamma such that all
// gamma * level[i] are (nearly) exact in fp16, stores those, and folds 1/gamma into the score
// scale and the output normalisation.
//
// Arithmetic.  K side: v_dot2_f32_f16 of the looked-up pair with the query pair, fp32
// accumulate, block scale applied once per 32 elements.  V side: fp32 accumulators; at k = 4 and
// k = 2 two tokens at a time, their codes merged nibble-wise so that one look-up returns the
// levels of one element for both tokens and one v_dot2_f32_f16 contracts them with the fp16 pair
// of weights p_t * scale (k = 3: v_fma_mix_f32 per element and token).  Softmax is the running-maximum form per wave:
// scores of a trip (64 or 128 tokens) are reduced to a wave maximum with DPP, the accumulators
// are rescaled only when the maximum grows (a wave-uniform branch), and the exponentials use
// exp2 with log2(e) folded into the score scale.  At the end of an item the next item's first
// loads are issued, then the 16 (or 32) token groups of each wave are summed with a
// reduce-scatter over lanes (v_permlane32_swap / v_permlane16_swap / DPP / ds_swizzle), the eight
// waves meet in 4 KiB of LDS, and the workgroup writes fp16 output or an fp32 partial
// (m, l, o[D]).  With split-K the workgroup that finishes an item's last partial (an integer
// ticket per batch*head, no floating-point atomics) combines all of them in an order fixed by
// its thread layout, so the result does not depend on which workgroup that was.
//
// Variants (template parameters of the one kernel): SPLIT as above; FUSE, the whole decode step
// of Sec. 3.2 in one launch -- the new token's rows are quantized in the kernel, appended to the
// cache and attended over; VARLEN, a length per sequence read from device memory.
#include "code_search.h"
#include "decode_common.h"
#include "nqkv_internal.h"
#include "scalar_read.h"

// Measurement build (-DNQKV_TIMELINE, see build.py --timeline): every wave records the 100 MHz
// real-time counter at eight points of an item's life and leaves them in the caller's workspace,
// 64 bytes per wave at byte offset kTimelineOffset + (item * 8 + wave) * 64, for items below
// kTimelineItems.  The stamps overwrite unused ticket counters (a call has at most 65535 of them and
// the configurations this is for use a few hundred), so such a build is for timing studies with
// fewer than 16384 (batch, head) pairs and a workspace of at least 1 MiB, and for nothing else.
#ifdef NQKV_TIMELINE
#define NQKV_STAMP(k_)                                     \
  do {                                                     \
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");     \
    timeline[k_] = __builtin_amdgcn_s_memrealtime();       \
  } while (0)
#else
#define NQKV_STAMP(k_) do { } while (0)
#endif

namespace nqkv {
namespace {

[[maybe_unused]] constexpr int kTimelineOffset = 65536, kTimelineItems = 1024;   // used by the measurement build only
constexpr int kWaves = 8;
constexpr int kThreads = 64 * kWaves;
constexpr int kRounds = 4;               // wave loads of K (and of V) in flight per trip

// ------------------------------------------------------------------ 3-bit codes
// A lane's 32 codes are a 96-bit stream, pair pr (elements 2 pr, 2 pr + 1) at bits [6 pr, 6 pr + 6):
// not byte aligned, and an address built by shift-and-mask costs two vector instructions per
// look-up.  Instead the stream is shifted right as a whole by 0, 6, 12 and 18 bits (three funnel
// shifts per version): in version v the pairs pr = v, v + 4, v + 8, v + 12 start at bits 0, 24, 48
// and 72 -- bytes 0 and 3 of dword 0, byte 2 of dword 1, byte 1 of dword 2 -- so one v_perm_b32
// forms each address, as for the other widths: 25 instructions for 16 look-ups instead of 34.  The
// two bits above a pair in its byte belong to the next pair; the table is indexed by the whole
// byte and ignores them (256 rows).  f(pr, address) is called once per pair.
template <class F>
__device__ __forceinline__ void for_each_pair_k3(const uint32_t (&w)[3], uint32_t lane_off, F&& f) {
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    uint32_t s0 = w[0], s1 = w[1], s2 = w[2];
    if (v > 0) {
      s0 = __builtin_amdgcn_alignbit(w[1], w[0], 6 * v);
      s1 = __builtin_amdgcn_alignbit(w[2], w[1], 6 * v);
      s2 = w[2] >> (6 * v);
    }
    f(v, row_addr<0>(s0, lane_off));
    f(v + 4, row_addr<3>(s0, lane_off));
    f(v + 8, row_addr<2>(s1, lane_off));
    f(v + 12, row_addr<1>(s2, lane_off));
  }
}

// The table for that: row = byte B (bits 6 and 7 ignored), 256 bytes apart, its first 128 bytes
// 32 copies of the dword {level[B & 7], level[(B >> 3) & 7]}; lane L reads copy L & 31.  Thread t
// writes copy t & 31 of rows (t >> 5) + 16 i: the low code follows from the thread index, the high
// code is (t >> 8) + 2 (i & 3).  Ends with a barrier.
__device__ __forceinline__ void build_lut_bytes_k3(const DecodeParams& p, uint32_t* smem) {
  const uint32_t copy = threadIdx.x & 31, e0 = threadIdx.x >> 5;       // e0 in [0, 16)
  const uint32_t lo = pick_level(p, e0 & 7, 8);
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const uint32_t hi_a = p.lut_levels[2 * (i & 3)], hi_b = p.lut_levels[2 * (i & 3) + 1];
    smem[(e0 + 16 * i) * 64 + copy] = lo | (((e0 >> 3) ? hi_b : hi_a) << 16);
  }
  __syncthreads();
}

// lut_levels[first + sel] for a constant `first` (a multiple of 2) and a wave-uniform sel in [0, 4),
// from scalar registers.  Indexed by a register, the kernel-argument array is read with a VECTOR
// load, and so is a select over constant indices (the compiler selects the address and loads
// afterwards): such a load queues behind the cache prefetches already in flight -- the memory
// counter is positional -- and the table build would wait for HBM.  The two dwords that hold the
// four candidates are therefore pinned in scalar registers as values before the selection.
__device__ __forceinline__ uint32_t uniform_level(const DecodeParams& p, int first, uint32_t sel) {
  uint32_t d0, d1;
  __builtin_memcpy(&d0, &p.lut_levels[first], 4);
  __builtin_memcpy(&d1, &p.lut_levels[(first + 2) & (kMaxLevels - 2)], 4);
  asm volatile("" : "+s"(d0), "+s"(d1));
  const uint32_t d = (sel & 2u) ? d1 : d0;
  return (sel & 1u) ? (d >> 16) : (d & 0xffffu);
}

// The table at k = 4: row = code byte B, 256 bytes apart, its first 128 bytes 32 copies of the dword
// {level[B & 15], level[B >> 4]}; lane L reads copy L & 31 (a 64-lane dword read takes two LDS
// clocks whatever it does, and 32 lanes on 32 distinct banks fit one of them: 32 copies are as
// conflict-free as 64 and take half the stores).  The copies of a row hold one and the same dword,
// so a thread writes four of them at a time: thread t takes low nibble t & 15, copies
// 4 ((t >> 4) & 7) .. + 3 and the four high nibbles (t >> 7) + 4 i -- 4 wide stores per thread
// where a dword at a time takes 32.  The high nibble is uniform over a wave: a scalar look-up.
// Ends with a barrier.
__device__ __forceinline__ void build_lut_k4(const DecodeParams& p, uint32_t* smem) {
  const uint32_t e_lo = threadIdx.x & 15, quad = (threadIdx.x >> 4) & 7;
  const uint32_t hi_base = __builtin_amdgcn_readfirstlane(threadIdx.x >> 7);       // 0..3
  const uint32_t lo = pick_level(p, e_lo, 16);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t e_hi = hi_base + 4 * i;
    const uint32_t v = lo | (uniform_level(p, 4 * i, hi_base) << 16);
    *reinterpret_cast<uint4*>(smem + (e_lo + 16 * e_hi) * 64 + quad * 4) = make_uint4(v, v, v, v);
  }
  __syncthreads();
}

// First link of a chain of v_dot2_f32_f16: the three-source form with a zero addend (written as
// an instruction because the compiler otherwise clears a register first and uses the
// accumulate-in-place form).
__device__ __forceinline__ float dot2_first(uint32_t a, uint32_t b) {
  float r;
  asm("v_dot2_f32_f16 %0, %1, %2, 0" : "=v"(r) : "v"(a), "v"(b));
  return r;
}

// ------------------------------------------------------------------ per-lane 32-element pieces
// K side: sum over the lane's 32 elements of q_d * level[code_d]
template <int KBITS>
__device__ __forceinline__ float k_dot(const uint32_t (&w)[KBITS], const uint32_t (&q2)[16],
                                       const char* lut, uint32_t lane_off) {
  float acc = 0.0f;
  if constexpr (KBITS == 4) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t a[4] = {row_addr<0>(w[i], lane_off), row_addr<1>(w[i], lane_off),
                             row_addr<2>(w[i], lane_off), row_addr<3>(w[i], lane_off)};
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        const uint32_t v = *reinterpret_cast<const uint32_t*>(lut + a[b]);
        if (i == 0 && b == 0) acc = dot2_first(v, q2[0]);
        else acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, v), __builtin_bit_cast(half2_t, q2[4 * i + b]), acc, false);
      }
    }
  } else if constexpr (KBITS == 2) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const uint32_t a[4] = {row_addr<0>(w[i], lane_off), row_addr<1>(w[i], lane_off),
                             row_addr<2>(w[i], lane_off), row_addr<3>(w[i], lane_off)};
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        const uint2 v = *reinterpret_cast<const uint2*>(lut + a[b]);
        if (i == 0 && b == 0) acc = dot2_first(v.x, q2[0]);
        else acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, v.x), __builtin_bit_cast(half2_t, q2[8 * i + 2 * b]), acc, false);
        acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, v.y), __builtin_bit_cast(half2_t, q2[8 * i + 2 * b + 1]), acc, false);
      }
    }
  } else {
    for_each_pair_k3(w, lane_off, [&](int pr, uint32_t addr) {
      const uint32_t v = *reinterpret_cast<const uint32_t*>(lut + addr);
      if (pr == 0) acc = dot2_first(v, q2[0]);
      else acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, v), __builtin_bit_cast(half2_t, q2[pr]), acc, false);
    });
  }
  return acc;
}

// V side: acc[e] += wgt * level[code_e]
template <int KBITS>
__device__ __forceinline__ void v_axpy(const uint32_t (&w)[KBITS], float wgt, float (&acc)[32],
                                       const char* lut, uint32_t lane_off) {
  if constexpr (KBITS == 4) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t a[4] = {row_addr<0>(w[i], lane_off), row_addr<1>(w[i], lane_off),
                             row_addr<2>(w[i], lane_off), row_addr<3>(w[i], lane_off)};
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        const half2_t h = __builtin_bit_cast(half2_t, *reinterpret_cast<const uint32_t*>(lut + a[b]));
        acc[8 * i + 2 * b + 0] = __builtin_fmaf((float)h.x, wgt, acc[8 * i + 2 * b + 0]);
        acc[8 * i + 2 * b + 1] = __builtin_fmaf((float)h.y, wgt, acc[8 * i + 2 * b + 1]);
      }
    }
  } else if constexpr (KBITS == 2) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const uint32_t a[4] = {row_addr<0>(w[i], lane_off), row_addr<1>(w[i], lane_off),
                             row_addr<2>(w[i], lane_off), row_addr<3>(w[i], lane_off)};
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        const uint2 v = *reinterpret_cast<const uint2*>(lut + a[b]);
        const half2_t x = __builtin_bit_cast(half2_t, v.x), y = __builtin_bit_cast(half2_t, v.y);
        const int e = 16 * i + 4 * b;
        acc[e + 0] = __builtin_fmaf((float)x.x, wgt, acc[e + 0]);
        acc[e + 1] = __builtin_fmaf((float)x.y, wgt, acc[e + 1]);
        acc[e + 2] = __builtin_fmaf((float)y.x, wgt, acc[e + 2]);
        acc[e + 3] = __builtin_fmaf((float)y.y, wgt, acc[e + 3]);
      }
    }
  } else {
    for_each_pair_k3(w, lane_off, [&](int pr, uint32_t addr) {
      const half2_t h = __builtin_bit_cast(half2_t, *reinterpret_cast<const uint32_t*>(lut + addr));
      acc[2 * pr + 0] = __builtin_fmaf((float)h.x, wgt, acc[2 * pr + 0]);
      acc[2 * pr + 1] = __builtin_fmaf((float)h.y, wgt, acc[2 * pr + 1]);
    });
  }
}

// V side, two tokens at a time: acc[e] += w(t0) * level[code(t0, e)] + w(t1) * level[code(t1, e)]
// with ONE v_dot2_f32_f16 per element, where the one-token form above spends one v_fma_mix per
// (token, element).  The code dwords of the two tokens are interleaved field by field first, a
// field being one code (F = k bits, mask M = the even fields of every byte):
//     a = (w0 & M) | ((w1 << F) & ~M)        even fields of t0, each followed by the same field of t1
//     b = ((w0 >> F) & M) | (w1 & ~M)        odd fields likewise
// (four instructions per dword pair), so that in `a` and `b` the code of an element of t0 is
// followed by the code of the SAME element of t1, and the byte-indexed table of the key side --
// which maps every field of a byte to its level, whatever the field means -- returns them side by
// side, {level of t0, level of t1}, ready to be contracted with the fp16 pair of weights.
// k = 4: a byte of `a` is element 2 j of both tokens, of `b` element 2 j + 1.  k = 2: a byte of `a`
// is elements 4 j and 4 j + 2 of both tokens (one 64-bit look-up, two contractions), of `b`
// elements 4 j + 1 and 4 j + 3.  The weights w = p * value scale are rounded to fp16 (round to
// nearest): a relative error of 2^-11 per term, of random sign.
template <int KBITS>
__device__ __forceinline__ void v_axpy_pair(const uint32_t (&w0)[KBITS], const uint32_t (&w1)[KBITS], half2_t wgt2,
                                            float (&acc)[32], const char* lut, uint32_t lane_off) {
  static_assert(KBITS == 4 || KBITS == 2, "3-bit codes do not align with bytes");
  constexpr uint32_t M = (KBITS == 4) ? 0x0f0f0f0fu : 0x33333333u;
#pragma unroll
  for (int i = 0; i < KBITS; ++i) {
    const uint32_t a = (w0[i] & M) | ((w1[i] << KBITS) & ~M);
    const uint32_t b = ((w0[i] >> KBITS) & M) | (w1[i] & ~M);
    const uint32_t aa[4] = {row_addr<0>(a, lane_off), row_addr<1>(a, lane_off), row_addr<2>(a, lane_off), row_addr<3>(a, lane_off)};
    const uint32_t ab[4] = {row_addr<0>(b, lane_off), row_addr<1>(b, lane_off), row_addr<2>(b, lane_off), row_addr<3>(b, lane_off)};
    if constexpr (KBITS == 4) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint32_t lo = *reinterpret_cast<const uint32_t*>(lut + aa[j]);
        const uint32_t hi = *reinterpret_cast<const uint32_t*>(lut + ab[j]);
        acc[8 * i + 2 * j + 0] = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, lo), wgt2, acc[8 * i + 2 * j + 0], false);
        acc[8 * i + 2 * j + 1] = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, hi), wgt2, acc[8 * i + 2 * j + 1], false);
      }
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint2 ev = *reinterpret_cast<const uint2*>(lut + aa[j]);
        const uint2 od = *reinterpret_cast<const uint2*>(lut + ab[j]);
        const int e = 16 * i + 4 * j;
        acc[e + 0] = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, ev.x), wgt2, acc[e + 0], false);
        acc[e + 2] = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, ev.y), wgt2, acc[e + 2], false);
        acc[e + 1] = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, od.x), wgt2, acc[e + 1], false);
        acc[e + 3] = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, od.y), wgt2, acc[e + 3], false);
      }
    }
  }
}

// The table at k = 2: row = code byte B with 2-bit fields c0..c3, 256 bytes apart: 32 copies of the
// eight bytes {level[c0], level[c1]}, {level[c2], level[c3]}; lane L reads copy L & 31 (a 64-lane
// 64-bit read takes four LDS clocks whatever it does, and 32 lanes on distinct bank pairs fit two of
// them: no conflicts, where 16 copies conflict two ways).  Thread t writes copies 2 (t & 15),
// 2 (t & 15) + 1 (one 128-bit store) of rows (t >> 4) + 32 i: c0 and c1 follow from the thread
// index, c2 = (t >> 8) + 2 (i & 1) and c3 = i >> 1 are uniform over a wave.  Ends with a barrier.
__device__ __forceinline__ void build_lut_k2(const DecodeParams& p, uint32_t* smem) {
  const uint32_t quad = threadIdx.x & 15, r0 = threadIdx.x >> 4;                 // r0 in [0, 32)
  const uint32_t c2_base = __builtin_amdgcn_readfirstlane(threadIdx.x >> 8);     // 0 or 1
  const uint32_t lo = pick_level(p, r0 & 3, 4) | (pick_level(p, (r0 >> 2) & 3, 4) << 16);
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const uint32_t hi = uniform_level(p, 2 * (i & 1), c2_base) | ((uint32_t)p.lut_levels[i >> 1] << 16);
    *reinterpret_cast<uint4*>(smem + (r0 + 32 * i) * 64 + quad * 4) = make_uint4(lo, hi, lo, hi);
  }
  __syncthreads();
}

// ------------------------------------------------------------------ in-wave reduce-scatter
// Sums acc[0..31] over the token groups of a wave (lanes with equal lane % LPT).  Each step
// halves the number of values a lane holds and sums across one lane bit:
//   bit 5: v_permlane32_swap, bit 4: v_permlane16_swap, bit 3: DPP row_ror:8, bit 2: ds_swizzle
//   xor 4, (LPT == 2 only) bit 1: DPP quad_perm xor 2.
// Afterwards a lane holds elements  e = 16 b5 + 8 b4 + 4 b3 + 2 b2 + i  (i = 0, 1; LPT == 4) or
// e = 16 b5 + 8 b4 + 4 b3 + 2 b2 + b1 (LPT == 2) of head-dim slice j = lane % LPT, where b_n is
// bit n of the lane index.
// The swaps are written as inline assembly: with the compiler builtin for these instructions
// the sum of the two results came out as (first + first) in this toolchain.  v_permlane32_swap
// exchanges lanes 32..63 of its first operand with lanes 0..31 of its second (v_permlane16_swap:
// odd 16-lane rows of the first with even rows of the second), so first + second afterwards is
// the sum over that lane bit, with the low half-lanes holding `a` and the high ones `b`.  The
// s_nop covers the wait states these instructions need after a VALU write of their operands.
__device__ __forceinline__ float swap32_add(float a, float b) {
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
  return a + b;
}
__device__ __forceinline__ float swap16_add(float a, float b) {
  asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1" : "+v"(a), "+v"(b));
  return a + b;
}
constexpr int kRowRor8 = 0x128;
constexpr int kSwizzleXor4 = 0x101F;

template <int LPT>
__device__ __forceinline__ void reduce_groups(const float (&acc)[32], uint32_t lane, float (&out)[2]) {
  float a16[16], a8[8], a4[4];
#pragma unroll
  for (int i = 0; i < 16; ++i) a16[i] = swap32_add(acc[i], acc[i + 16]);
#pragma unroll
  for (int i = 0; i < 8; ++i) a8[i] = swap16_add(a16[i], a16[i + 8]);
  const bool b3 = lane & 8, b2 = lane & 4, b1 = lane & 2;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float send = b3 ? a8[i] : a8[i + 4], keep = b3 ? a8[i + 4] : a8[i];
    a4[i] = keep + dpp_f<kRowRor8>(send);
  }
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const float send = b2 ? a4[i] : a4[i + 2], keep = b2 ? a4[i + 2] : a4[i];
    out[i] = keep + __builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, send), kSwizzleXor4));
  }
  if (LPT == 2) {
    const float send = b1 ? out[0] : out[1], keep = b1 ? out[1] : out[0];
    out[0] = keep + dpp_f<kQuadXor2>(send);
  }
}

// ------------------------------------------------------------------ main kernel
// grid: x = workgroups, each taking items i = blockIdx.x, + gridDim.x, ...; item i -> (bh = i / splits, split = i % splits)
// SPLIT: sequences are cut into p.splits > 1 items whose partial results are combined by the
// workgroup that finishes last; without it (p.splits == 1) that code and the item -> (sequence,
// split) division are compiled out.
// VARLEN: every sequence of the batch has its own number of cached tokens, read from device
// memory (p.seq_lens[b], clamped to [0, p.max_len]); the split geometry is laid out for
// p.max_len and each item keeps the part of its range that lies inside its sequence.
// PAGED (with VARLEN): the cache is a pool of pages behind a block table; token ranges stay
// logical and every trip translates its start token to a page (see page_rows).
// FUSE: the whole decode step of the paper in one launch -- items cover the tokens already
// cached, rows [0, pos); the last wave of each sequence's last item quantizes the new token's
// key and value rows (same code search as the quantizer), stores their codes and scales at row
// pos, and adds the token to its softmax straight from registers.
template <int KBITS, int D, int BLK, bool FUSE, bool SPLIT, bool VARLEN, bool PAGED>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_num_vgpr(128), amdgpu_waves_per_eu(4, 4))) void decode_kernel(const DecodeParams p) {   // 128 VGPRs, four waves per SIMD: two workgroups per CU
  constexpr int LPT = D / 32;             // lanes per token
  constexpr int TPR = 64 / LPT;           // tokens per wave load
  constexpr int CHUNK = kRounds * TPR;    // tokens per wave trip
  constexpr int NB = D / BLK;
  constexpr int ROW = LPT * KBITS;        // dwords of codes per token
  // One LDS object, the small arrays first: everything but the table then lies below 64 KiB,
  // within reach of the 16-bit offset field of the LDS instructions.  (As separate variables the
  // compiler put the table first, and every fixed address above 64 KiB cost a register that
  // stayed live around the whole item loop.)
  struct Lds {
    float xw[kWaves][D];                            // per-wave partial outputs
    float wave_m[kWaves], wave_l[kWaves];
    uint32_t ticket;
    uint2 cells[FUSE ? 128 : 1];                    // FUSE: code-search cell table
    uint32_t new_codes[FUSE ? 2 : 1][ROW];          // packed codes of the new token's K and V rows
    uint32_t new_scales[FUSE ? 2 : 1][NB];          // and their block scales (fp16 bits)
    __attribute__((aligned(256))) uint32_t lut[kLutWords];
  };
  __shared__ Lds lds;
  uint32_t* const smem = lds.lut;
  auto& xw = lds.xw;
  auto& wave_m = lds.wave_m;
  auto& wave_l = lds.wave_l;
  uint32_t& ticket_sh = lds.ticket;
  auto& cells = lds.cells;
  auto& new_codes = lds.new_codes;
  auto& new_scales = lds.new_scales;

  const char* lut = reinterpret_cast<const char*>(smem);
  const uint32_t lane = threadIdx.x & 63;
  // the wave index as a scalar, so that everything derived from it (token ranges, the full-trip
  // test) is uniform control flow for the compiler
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint32_t j = lane % LPT, g = lane / LPT;
  // this lane's copy inside a table row: 32 copies of a dword (k = 3, 4) or of a dword pair (k = 2)
  const uint32_t lane_off = (lane & 31) << (KBITS == 2 ? 3 : 2);
  const int32_t stride = kWaves * CHUNK;

  uint32_t kw[kRounds][KBITS], vw[kRounds][KBITS];
  uint16_t ksc[kRounds], vsc[kRounds];
  uint32_t q2[16];

  // Item geometry.  Split sp of a sequence covers sp * split_base + min(sp, split_rem) onwards,
  // split_base (+1 for the first split_rem splits) tokens: never empty.  Token counts below are
  // relative to the item's first token and fit 32 bits with room to spare (host-checked).
  constexpr uint32_t kRowBytes = ROW * 4, kScaleRowBytes = NB * 2;
  const uint32_t code_voff = g * kRowBytes + j * (KBITS * 4);            // this lane's slice of a token row
  const uint32_t scale_voff = g * kScaleRowBytes + ((j * 32) / BLK) * 2;
  uint32_t bh = 0, sp = 0;
  int32_t n_tok = 0, base = 0;      // tokens in the item; this wave's current trip start (item-relative)
  int32_t front = 0;                // rows taken in before the item's first token, masked (see set_item)
  int64_t pos = 0;                  // FUSE and VARLEN: the sequence's own row for the new token (else p.pos)
  __amdgpu_buffer_rsrc_t kc_r, vc_r, ks_r, vs_r;
  // PAGED: the item's sequence, head and first token (logical), and the pool rows / row count
  // of the trip whose K loads were issued last (its V loads follow at the top of the trip)
  uint32_t item_b = 0, item_h = 0;
  int32_t item_t0 = 0, trip_left = 0;
  int64_t trip_rows = 0;
  __amdgpu_buffer_rsrc_t kn_r, vn_r;      // FUSE: the new token's rows, empty for waves that do not take it
  uint32_t newx[4] = {0, 0, 0, 0};        // FUSE: this lane's 16-byte chunk of those rows
  auto set_item = [&](uint32_t item) {
    if (SPLIT) {
      bh = item / (uint32_t)p.splits;
      sp = item - bh * (uint32_t)p.splits;
    } else {
      bh = item; sp = 0;
    }
    const int64_t t0 = (int64_t)sp * p.split_base + min((int32_t)sp, p.split_rem);
    n_tok = p.split_base + ((int32_t)sp < p.split_rem ? 1 : 0);
    uint32_t b = 0, h = 0;
    int64_t row0 = (int64_t)bh * p.cap_tokens + t0;
    if (VARLEN) {
      b = bh / (uint32_t)p.H; h = bh - b * (uint32_t)p.H;
      if (p.longest_first) {
        // b so far is a rank: take the sequence whose length has that rank (ties by index).  Lane l
        // holds the length of sequence l (at most 64 of them); its rank is the number of sequences
        // that come before it.  Items are dispatched in index order, so the long sequences start
        // first and the short ones fill the tail of the grid.
        const uint32_t nb = (uint32_t)p.n_seqs;
        int32_t len_l = -1;
        if (lane < nb) len_l = min(max(p.seq_lens[lane], 0), p.max_len);
        uint32_t before = 0;
        for (uint32_t s = 0; s < nb; ++s) {
          const int32_t len_s = __builtin_amdgcn_readlane(len_l, (int)s);
          before += (len_s > len_l || (len_s == len_l && s < lane)) ? 1u : 0u;
        }
        const uint64_t hit = __builtin_amdgcn_ballot_w64(lane < nb && before == b);
        b = hit ? (uint32_t)__builtin_ctzll(hit) : b;       // exactly one lane: the ranks are a permutation
        bh = b * (uint32_t)p.H + h;
        row0 = (int64_t)bh * p.cap_tokens + t0;
      }
      const int32_t len = min(max(scalar_read(p.seq_lens + b), 0), p.max_len);     // whatever the array holds, stay inside the cache
      n_tok = min(n_tok, max(len - (int32_t)t0, 0));
      pos = len;
      if (PAGED) { item_b = b; item_h = h; item_t0 = (int32_t)t0; }
    }
    // Wave loads cover 512 to 1024 contiguous bytes; they are cheapest when they start on a
    // 128-byte line.  Whether the item's first row does depends on the caller's capacity (the
    // distance between slabs) and on where a split begins.  When it does not, and whole rows fit
    // in between, the item starts up to 7 rows EARLIER -- rows of the same tensor, inside the line
    // its first row shares anyway -- and the tokens taken in are masked out of the softmax in the
    // item's first trip.  (Measured at B16 H56 D128 S16384, 4 bits, capacity 16385, where every
    // other slab is 64 bytes off: 407 -> 374 us per launch behind the quantizer, 332 -> 307 us back to back.)
    front = 0;
    if constexpr (!PAGED && 128 % kRowBytes == 0) {
      const uint32_t past_line = (uint32_t)(reinterpret_cast<uintptr_t>(p.k_codes) + (uint64_t)row0 * kRowBytes) & 127u;
      front = n_tok > 0 ? (int32_t)min((int64_t)(past_line / kRowBytes), row0) : 0;
      row0 -= front;
      n_tok += front;
    }
    base = (int32_t)wave * CHUNK;
    kc_r = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(p.k_codes) + row0 * kRowBytes, 0, n_tok * (int)kRowBytes, kBufferFlags);
    vc_r = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(p.v_codes) + row0 * kRowBytes, 0, n_tok * (int)kRowBytes, kBufferFlags);
    ks_r = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.k_scales) + row0 * NB, 0, n_tok * (int)kScaleRowBytes, kBufferFlags);
    vs_r = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.v_scales) + row0 * NB, 0, n_tok * (int)kScaleRowBytes, kBufferFlags);
    if (FUSE) {
      if (!VARLEN) { b = bh / (uint32_t)p.H; h = bh - b * (uint32_t)p.H; }
      const int64_t off = (int64_t)b * p.new_stride_b + (int64_t)h * p.new_stride_h;
      const int bytes = ((!SPLIT || sp == (uint32_t)p.splits - 1u) && wave == kWaves - 1) ? D * 2 : 0;
      kn_r = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.k_new) + off, 0, bytes, kBufferFlags);
      vn_r = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.v_new) + off, 0, bytes, kBufferFlags);
    }
  };
  // FUSE: one lane per 16-byte chunk -- lanes [0, D/8) take the key row, the next D/8 the value
  // row.  The range check does the predication: a lane outside its row (and every lane of a wave
  // whose descriptors are empty) reads zeros, so the two loads are issued unconditionally, like
  // the trip loads, and sit in the same prefetch slot as the first K trip.
  auto load_new = [&]() {
    uint32_t a[4], c[4];
    load_codes<4>(kn_r, lane * 16u, 0, a);
    constexpr uint32_t CPR = D / 8;
    load_codes<4>(vn_r, lane >= CPR ? (lane - CPR) * 16u : 0x40000000u, 0, c);     // far out of range, no wrap
#pragma unroll
    for (int i = 0; i < 4; ++i) newx[i] = a[i] | c[i];
  };

  // Loads of one trip starting at item-relative token tb (uniform).  The trip offset goes into
  // voffset, which is what the hardware range-checks: tokens past the end of the item (the
  // ragged last trip, or a whole trip that does not exist) read zeros and touch no memory.  That
  // lets every trip issue exactly the same loads unconditionally, which matters because the
  // memory counter is positional: loads issued under a branch make the compiler wait for the
  // worst case at the join.
  auto load_trip = [&](__amdgpu_buffer_rsrc_t codes, __amdgpu_buffer_rsrc_t scales, int32_t tb,
                       uint32_t (&w)[kRounds][KBITS], uint16_t (&sc)[kRounds]) {
    const uint32_t cv = code_voff + (uint32_t)tb * kRowBytes;
    const uint32_t sv = scale_voff + (uint32_t)tb * kScaleRowBytes;
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
      load_codes<KBITS>(codes, cv + r * TPR * kRowBytes, 0, w[r]);
      sc[r] = __builtin_amdgcn_raw_buffer_load_b16(scales, sv + r * TPR * kScaleRowBytes, 0, 0);
    }
  };
  // PAGED: pool rows of the trip that starts at item-relative token tb.  Items start at multiples
  // of the page size and trips at multiples of CHUNK, which divides it, so a trip never straddles
  // two pages.  Table index and entry are clamped: nothing the table holds (and no trip past the
  // end of the sequence, whose row count is 0) can address memory outside the pool.
  auto page_rows = [&](int32_t tb) {
    const int32_t tok = item_t0 + tb;
    const int32_t lp = min(tok >> p.page_shift, p.table_stride - 1);
    const int32_t phys = min(max(scalar_read(p.block_table + ((int64_t)item_b * p.table_stride + lp)), 0), p.num_pages - 1);
    trip_rows = ((((int64_t)phys * p.H + item_h)) << p.page_shift) + (tok & ((1 << p.page_shift) - 1));
    // (the clamp selects as a vector instruction; without the readfirstlane the descriptors built
    // from it would count as non-uniform and every load would run in a make-uniform loop)
    trip_left = __builtin_amdgcn_readfirstlane(min(max(n_tok - tb, 0), CHUNK));
  };
  auto load_rows = [&](const uint8_t* codes, const uint16_t* scales,
                       uint32_t (&w)[kRounds][KBITS], uint16_t (&sc)[kRounds]) {
    const __amdgpu_buffer_rsrc_t cr = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(codes) + trip_rows * kRowBytes, 0, trip_left * (int)kRowBytes, kBufferFlags);
    const __amdgpu_buffer_rsrc_t sr = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t*>(scales) + trip_rows * NB, 0, trip_left * (int)kScaleRowBytes, kBufferFlags);
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
      load_codes<KBITS>(cr, code_voff + r * TPR * kRowBytes, 0, w[r]);
      sc[r] = __builtin_amdgcn_raw_buffer_load_b16(sr, scale_voff + r * TPR * kScaleRowBytes, 0, 0);
    }
  };
  // K loads of the trip at tb; V loads of the trip whose K loads went out last
  auto load_k = [&](int32_t tb) {
    if constexpr (PAGED) { page_rows(tb); load_rows(p.k_codes, p.k_scales, kw, ksc); }
    else load_trip(kc_r, ks_r, tb, kw, ksc);
  };
  auto load_v = [&](int32_t tb) {
    if constexpr (PAGED) load_rows(p.v_codes, p.v_scales, vw, vsc);
    else load_trip(vc_r, vs_r, tb, vw, vsc);
  };
  auto load_q = [&]() {
    const uint4* qp = reinterpret_cast<const uint4*>(p.q + (int64_t)bh * D + j * 32);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint4 v = qp[i];
      q2[4 * i] = v.x; q2[4 * i + 1] = v.y; q2[4 * i + 2] = v.z; q2[4 * i + 3] = v.w;
    }
  };

  // The first item's K loads and query slice go out before anything else, so HBM latency
  // overlaps the table build.
  uint32_t item = blockIdx.x;
#ifdef NQKV_TIMELINE
  uint64_t timeline[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#endif
  NQKV_STAMP(0);                       // the wave is running
  // FUSE: lane l fetches entry l of the code-search cell table.  These are vector loads from the
  // kernel arguments; they go out first so that waiting for them (the memory counter is
  // positional) never means waiting for the cache prefetches behind them.
  uint32_t cell_thr = 0, cell_below = 0;
  if (FUSE) { cell_thr = p.cell_thr[lane]; cell_below = p.cell_below[lane]; }
  set_item(item);
  load_k(base);
  load_q();
  if (FUSE) load_new();
  NQKV_STAMP(1);                       // first loads issued
  if constexpr (KBITS == 2) build_lut_k2(p, smem);          // (each ends with a barrier)
  else if constexpr (KBITS == 3) build_lut_bytes_k3(p, smem);
  else build_lut_k4(p, smem);
  NQKV_STAMP(2);                       // table built
  if (FUSE && wave == kWaves - 1) {
    // only this wave searches codes: it stages the table for itself, no barrier needed (LDS
    // operations of one wave complete in order)
    cells[lane] = make_uint2(cell_thr, cell_below);
    if (lane == 0) cells[code_search::kCells - 1] = make_uint2(p.cell_thr[code_search::kCells - 1], p.cell_below[code_search::kCells - 1]);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  }
  // Make the query registers "arrived" here, outside the trip loop: otherwise the wait for
  // them is re-imposed at the top of every trip (it is pending on the loop-entry path only), and
  // because the memory counter is positional that stalls each trip on its own fresh V loads.
  auto settle_q = [&]() {
#pragma unroll
    for (int i = 0; i < 16; ++i) asm volatile("" ::"v"(q2[i]));
  };
  settle_q();

  while (true) {
    float acc[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) acc[i] = 0.0f;
    float m_run = kNoScore;    // wave-uniform, log2 domain
    float l_run = 0.0f;        // per lane; every lane of a token group adds the same p

    if (FUSE && (!SPLIT || sp == (uint32_t)p.splits - 1u) && wave == kWaves - 1) {
      // ---- the token of this step: quantize, append, attend -- before this wave's share of
      // the cached tokens, while the accumulators are not live yet.  One lane per 16-byte chunk
      // (fetched by load_new), so the whole code search is one chunk deep.
      constexpr uint32_t CPR = D / 8;         // chunks per row
      constexpr uint32_t LPB = BLK / 8;       // lanes per quantization block (8 or 16: inside a DPP row)
      // an opaque copy of the lane index: everything below is derived from it, so the compiler
      // cannot hoist these address computations out of this block, where their registers would
      // cost the streaming loop its occupancy
      __builtin_amdgcn_s_setprio(3);           // one wave's serial chain: do not queue behind the streaming waves
      uint32_t ql = lane;
      asm volatile("" : "+v"(ql));
      const uint32_t t = ql / CPR, c = ql % CPR;          // tensor (0 key, 1 value), chunk in the row
      const bool mine = t < 2;
      const uint4 x = make_uint4(newx[0], newx[1], newx[2], newx[3]);    // zeros where !mine
      const uint32_t M = 0x7fff7fffu;
      const uint32_t a2 = code_search::pk_max_u16(code_search::pk_max_u16(x.x & M, x.y & M),
                                                  code_search::pk_max_u16(x.z & M, x.w & M));
      uint32_t s_bits = max(a2 & 0xffffu, a2 >> 16);
      s_bits = max(s_bits, code_search::dpp<code_search::kQuadXor1>(s_bits));
      s_bits = max(s_bits, code_search::dpp<code_search::kQuadXor2>(s_bits));
      s_bits = max(s_bits, code_search::dpp<code_search::kRowHalfMirror>(s_bits));
      if (LPB == 16) s_bits = max(s_bits, code_search::dpp<code_search::kRowMirror>(s_bits));
      const uint32_t code = code_search::encode_chunk<KBITS, true>(x, s_bits, LevelTable{}, cells);
      if (mine) {
        // the LDS image of each row has the layout of a cache row: chunk c at byte c * KBITS
        uint8_t* img = reinterpret_cast<uint8_t*>(&new_codes[t][0]) + c * KBITS;
        if constexpr (KBITS == 4) {
          *reinterpret_cast<uint32_t*>(img) = code;
        } else if constexpr (KBITS == 2) {
          *reinterpret_cast<uint16_t*>(img) = (uint16_t)code;
        } else {
          img[0] = (uint8_t)code; img[1] = (uint8_t)(code >> 8); img[2] = (uint8_t)(code >> 16);
        }
        if (c % LPB == 0) new_scales[t][c / LPB] = s_bits;
      }
      // written and read by different lanes of this one wave: LDS operations of a wave complete
      // in order, the fence keeps the compiler from reordering them
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      uint32_t nk[KBITS], nv[KBITS];
      uint32_t nks = 0, nvs = 0;
#pragma unroll
      for (int i = 0; i < KBITS; ++i) { nk[i] = 0; nv[i] = 0; }
      if (ql < (uint32_t)LPT) {                 // token group 0: lane j owns 32 elements of each row
#pragma unroll
        for (int i = 0; i < KBITS; ++i) {
          nk[i] = new_codes[0][ql * KBITS + i];
          nv[i] = new_codes[1][ql * KBITS + i];
        }
        nks = new_scales[0][(ql * 32) / BLK];
        nvs = new_scales[1][(ql * 32) / BLK];
      }
      float part = k_dot<KBITS>(nk, q2, lut, lane_off);
      part *= (float)__builtin_bit_cast(_Float16, (unsigned short)nks);
      part += dpp_f<kQuadXor1>(part);
      if (LPT == 4) part += dpp_f<kQuadXor2>(part);
      const float z = (g == 0) ? part * p.scale_log2e : -INFINITY;
      m_run = wave_max(z);                                   // finite: group 0 holds a real score
      const float pn = __builtin_amdgcn_exp2f(z - m_run);    // 1 for the token's lanes, 0 elsewhere
      l_run = pn;
      v_axpy<KBITS>(nv, pn * (float)__builtin_bit_cast(_Float16, (unsigned short)nvs), acc, lut, lane_off);
      __builtin_amdgcn_s_setprio(0);
    }

    NQKV_STAMP(3);                     // trips begin
    for (; base < n_tok; base += stride) {
      const int32_t left = n_tok - base;      // tokens of the item from this trip on (uniform)
      load_v(base);

      // scores of this trip's tokens (log2 domain)
      float z[kRounds];
#pragma unroll
      for (int r = 0; r < kRounds; ++r) {
        float part = k_dot<KBITS>(kw[r], q2, lut, lane_off);
        // (an fma with a zero addend: it takes the fp16 scale as it is, where a multiply needs a conversion first)
        part = __builtin_fmaf(part, (float)__builtin_bit_cast(_Float16, ksc[r]), 0.0f);
        part += dpp_f<kQuadXor1>(part);
        if (LPT == 4) part += dpp_f<kQuadXor2>(part);
        z[r] = part * p.scale_log2e;
      }
      if (left < CHUNK || (front != 0 && base == 0)) {
        // the ragged last trip of the item (a uniform branch): tokens past the end read as zero codes
        // and zero scales, a score of 0, and must not enter the softmax; nor must the rows taken in
        // before the item's first token (first trip only: they are fewer than one round)
#pragma unroll
        for (int r = 0; r < kRounds; ++r) z[r] = ((int32_t)g < left - r * TPR) ? z[r] : -INFINITY;
        if (base == 0) {
          // (their value scales are whatever memory holds there, possibly not even finite: a zero
          // weight times such a scale must not reach the accumulators)
          z[0] = ((int32_t)g >= front) ? z[0] : -INFINITY;
          vsc[0] = ((int32_t)g >= front) ? vsc[0] : (uint16_t)0;
        }
      }
      float m_trip = fmaxf(z[0], z[1]);
#pragma unroll
      for (int r = 2; r < kRounds; r += 2) m_trip = fmaxf(m_trip, fmaxf(z[r], z[r + 1]));
      m_trip = wave_max<LPT>(m_trip);          // the LPT lanes of a token hold the same scores
      if (m_trip > m_run) {            // uniform across the wave
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_trip);
#pragma unroll
        for (int i = 0; i < 32; ++i) acc[i] *= alpha;
        l_run *= alpha;
        m_run = m_trip;
      }
      float pw[kRounds];
#pragma unroll
      for (int r = 0; r < kRounds; ++r) {
        pw[r] = __builtin_amdgcn_exp2f(z[r] - m_run);
        l_run += pw[r];
      }

      load_k(base + stride);     // past the end on the last trip: reads zeros

      if constexpr (KBITS == 3) {
#pragma unroll
        for (int r = 0; r < kRounds; ++r) {
          const float wgt = __builtin_fmaf(pw[r], (float)__builtin_bit_cast(_Float16, vsc[r]), 0.0f);
          v_axpy<KBITS>(vw[r], wgt, acc, lut, lane_off);
        }
      } else {
        // two tokens per step: one v_dot2 per element instead of two v_fma_mix
#pragma unroll
        for (int r = 0; r < kRounds; r += 2) {
          const float w_a = __builtin_fmaf(pw[r], (float)__builtin_bit_cast(_Float16, vsc[r]), 0.0f);
          const float w_b = __builtin_fmaf(pw[r + 1], (float)__builtin_bit_cast(_Float16, vsc[r + 1]), 0.0f);
          const half2_t wgt2 = {(_Float16)w_a, (_Float16)w_b};
          v_axpy_pair<KBITS>(vw[r], vw[r + 1], wgt2, acc, lut, lane_off);
        }
      }
    }

    NQKV_STAMP(4);                     // trips end
    // ---- this item is streamed; remember where its result goes, then start the next item's
    // first K loads so that they fly during the merge
    const uint32_t cur_bh = bh, cur_sp = sp;
    const int64_t cur_pos = pos;
    const uint32_t next_item = item + gridDim.x;
    const bool more = next_item < (uint32_t)p.n_items;
    if (more) {
      set_item(next_item);
      load_k(base);
      load_q();
      if (FUSE) load_new();
    }

    // ---- merge: token groups inside each wave, then the eight waves through LDS.
    // Everything here is addressed from an opaque copy of the thread index: derived from
    // threadIdx.x directly, these item-invariant addresses would be hoisted out of the item loop
    // and sit in registers through the streaming loop, which needs every one it can get.
    uint32_t tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const uint32_t mlane = tid & 63;
    float red[2];
    reduce_groups<LPT>(acc, mlane, red);
    const float l_wave = wave_sum(l_run) * (1.0f / LPT);
    {
      const uint32_t mj = mlane % LPT;
      const uint32_t e = ((mlane >> 5) & 1) * 16 + ((mlane >> 4) & 1) * 8 + ((mlane >> 3) & 1) * 4 + ((mlane >> 2) & 1) * 2;
      if (LPT == 4) {
        xw[wave][mj * 32 + e] = red[0];
        xw[wave][mj * 32 + e + 1] = red[1];
      } else {
        xw[wave][mj * 32 + e + ((mlane >> 1) & 1)] = red[0];
      }
      if (mlane == 0) { wave_m[wave] = m_run; wave_l[wave] = l_wave; }
    }
    __syncthreads();
    if (FUSE && (!SPLIT || cur_sp == (uint32_t)p.splits - 1u)) {
      // Append: the LDS images of the new token's rows go to cache row pos.  Done here rather
      // than where they are produced because stores share the loads' in-order memory counter:
      // issued ahead of the streaming loop, their acknowledgements would hold up its first trip.
      int64_t row = (int64_t)cur_bh * p.cap_tokens + (VARLEN ? cur_pos : p.pos);
      if (PAGED) {                                    // the row's page comes from the table
        const uint32_t cb = cur_bh / (uint32_t)p.H, ch = cur_bh - cb * (uint32_t)p.H;
        const int32_t lp = min((int32_t)(cur_pos >> p.page_shift), p.table_stride - 1);
        const int32_t phys = min(max(scalar_read(p.block_table + ((int64_t)cb * p.table_stride + lp)), 0), p.num_pages - 1);
        row = ((((int64_t)phys * p.H + ch)) << p.page_shift) + (cur_pos & ((1 << p.page_shift) - 1));
      }
      if (tid < 2u * ROW) {
        const uint32_t t = tid / ROW, w = tid % ROW;
        uint32_t* dst = reinterpret_cast<uint32_t*>(const_cast<uint8_t*>(t ? p.v_codes : p.k_codes)) + row * ROW + w;
        *dst = new_codes[t][w];
      } else if (tid < 2u * ROW + 2u * NB) {
        const uint32_t t = (tid - 2u * ROW) / NB, w = (tid - 2u * ROW) % NB;
        const_cast<uint16_t*>(t ? p.v_scales : p.k_scales)[row * NB + w] = (uint16_t)new_scales[t][w];
      }
    }
    NQKV_STAMP(5);                     // waves merged (past the barrier)
    float m_all = wave_m[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) m_all = fmaxf(m_all, wave_m[w]);
    float l_all = 0.0f, o = 0.0f;
    if (tid < D) {
#pragma unroll
      for (int w = 0; w < kWaves; ++w) {
        const float f = __builtin_amdgcn_exp2f(wave_m[w] - m_all);   // 0 for a wave that saw no token
        l_all += wave_l[w] * f;
        o += xw[w][tid] * f;
      }
      if (!SPLIT) {
        p.out[(int64_t)cur_bh * D + tid] = __builtin_bit_cast(unsigned short, (_Float16)(o * p.inv_gamma / l_all));
      } else {
        // Partials travel between workgroups, possibly on different XCDs whose L2 caches are not
        // coherent with each other: write them through (agent-scope stores) rather than paying
        // for a whole-L2 write-back fence per item.
        uint32_t* ws = reinterpret_cast<uint32_t*>(p.partials + ((int64_t)cur_bh * p.splits + cur_sp) * (D + 2));
        store_agent(ws + 2 + tid, o);
        if (tid == 0) { store_agent(ws, m_all); store_agent(ws + 1, l_all); }
      }
    }
    if (SPLIT) {
      // Once every store above is acknowledged, take a ticket; the workgroup holding the last
      // ticket of this (b,h) combines all partials in split order (reading them past the
      // caches) and re-arms the ticket counter.
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
      if (tid == 0) ticket_sh = __hip_atomic_fetch_add(p.tickets + cur_bh, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __syncthreads();
      // A ticket this call cannot have handed out: the counter did not start at zero (a workspace
      // that was never cleared, or clobbered since).  Leave a mark that the host can ask for.
      NQKV_STAMP(6);                   // partial result published, ticket taken
      if (ticket_sh >= (uint32_t)p.splits && tid == 0)
        __hip_atomic_fetch_or(p.tickets + kWorkspaceStatusWord, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (ticket_sh == (uint32_t)p.splits - 1u) {           // uniform over the workgroup
        // All 512 threads combine: thread (grp, d) folds the partials of splits grp, grp + G, ...
        // for output element d, four splits per trip so that their loads (which bypass the
        // caches, a full memory round trip each) are in flight together; the G group results
        // then merge through LDS exactly like the eight waves above.  The order of the folds is
        // fixed by this layout, not by which workgroup arrives last: equal inputs, equal bits.
        constexpr uint32_t G = kThreads / D, U = 4;
        const uint32_t grp = tid / D, d = tid % D;
        const uint32_t* ws = reinterpret_cast<const uint32_t*>(p.partials + (int64_t)cur_bh * p.splits * (D + 2));
        float mm = -INFINITY, ll = 0.0f, oo = 0.0f;
        for (uint32_t s0 = grp; s0 < (uint32_t)p.splits; s0 += G * U) {
          float ms[U], ls[U], os[U];
#pragma unroll
          for (uint32_t u = 0; u < U; ++u) {
            const uint32_t s2 = min(s0 + u * G, (uint32_t)p.splits - 1u);      // clamped: always a valid record
            const uint32_t* rec = ws + s2 * (D + 2);
            ms[u] = load_agent(rec);
            ls[u] = load_agent(rec + 1);
            os[u] = load_agent(rec + 2 + d);
          }
#pragma unroll
          for (uint32_t u = 0; u < U; ++u) {
            const float m_s = (s0 + u * G < (uint32_t)p.splits) ? ms[u] : -INFINITY;   // a clamped duplicate weighs 0
            const float m_new = fmaxf(mm, m_s);                 // finite: every stored m is (kNoScore at least)
            const float f_old = __builtin_amdgcn_exp2f(mm - m_new), f_s = __builtin_amdgcn_exp2f(m_s - m_new);
            ll = ll * f_old + ls[u] * f_s;
            oo = oo * f_old + os[u] * f_s;
            mm = m_new;
          }
        }
        xw[grp][d] = oo;
        if (d == 0) { wave_m[grp] = mm; wave_l[grp] = ll; }
        __syncthreads();
        if (tid < D) {
          float m_fin = wave_m[0];
#pragma unroll
          for (uint32_t g2 = 1; g2 < G; ++g2) m_fin = fmaxf(m_fin, wave_m[g2]);
          float l_fin = 0.0f, o_fin = 0.0f;
#pragma unroll
          for (uint32_t g2 = 0; g2 < G; ++g2) {
            const float f = __builtin_amdgcn_exp2f(wave_m[g2] - m_fin);       // 0 for a group without splits
            l_fin += wave_l[g2] * f;
            o_fin += xw[g2][tid] * f;
          }
          p.out[(int64_t)cur_bh * D + tid] = __builtin_bit_cast(unsigned short, (_Float16)(o_fin * p.inv_gamma / l_fin));
        }
        if (tid == 0) __hip_atomic_store(p.tickets + cur_bh, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
#ifdef NQKV_TIMELINE
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    NQKV_STAMP(7);                     // output (or the combined result) stored and acknowledged
    if (lane == 0 && p.tickets && item < (uint32_t)kTimelineItems) {
      unsigned long long* rec = reinterpret_cast<unsigned long long*>(reinterpret_cast<char*>(p.tickets) + kTimelineOffset) +
                                ((size_t)item * kWaves + wave) * 8;
      for (int k_ = 0; k_ < 8; ++k_) rec[k_] = timeline[k_];
    }
#endif
    settle_q();           // before the exit test, so that every path back to the loop head has it
    if (!more) break;
    item = next_item;
    __syncthreads();      // xw / wave_m / ticket_sh are reused by the next item
  }
}

template <int KBITS, int D, int BLK, bool VARLEN, bool PAGED>
hipError_t launch_var(const DecodeParams& p, bool fuse, hipStream_t stream) {
  const int wgs = p.n_items < p.max_workgroups ? p.n_items : p.max_workgroups;
  const dim3 grid((unsigned)wgs), block(kThreads);
  const bool split = p.splits > 1;
  if (fuse && split)       hipLaunchKernelGGL((decode_kernel<KBITS, D, BLK, true, true, VARLEN, PAGED>), grid, block, 0, stream, p);
  else if (fuse)           hipLaunchKernelGGL((decode_kernel<KBITS, D, BLK, true, false, VARLEN, PAGED>), grid, block, 0, stream, p);
  else if (split)          hipLaunchKernelGGL((decode_kernel<KBITS, D, BLK, false, true, VARLEN, PAGED>), grid, block, 0, stream, p);
  else                     hipLaunchKernelGGL((decode_kernel<KBITS, D, BLK, false, false, VARLEN, PAGED>), grid, block, 0, stream, p);
  return hipGetLastError();
}

template <int KBITS, int D, int BLK>
hipError_t launch_one(const DecodeParams& p, bool fuse, hipStream_t stream) {
  if (p.block_table) return launch_var<KBITS, D, BLK, true, true>(p, fuse, stream);
  return p.seq_lens ? launch_var<KBITS, D, BLK, true, false>(p, fuse, stream)
                    : launch_var<KBITS, D, BLK, false, false>(p, fuse, stream);
}

template <int KBITS>
hipError_t launch_k(const DecodeParams& p, int D, int blk, bool fuse, hipStream_t stream) {
  if (D == 64 && blk == 64) return launch_one<KBITS, 64, 64>(p, fuse, stream);
  if (D == 128 && blk == 64) return launch_one<KBITS, 128, 64>(p, fuse, stream);
  if (D == 128 && blk == 128) return launch_one<KBITS, 128, 128>(p, fuse, stream);
  return hipErrorInvalidValue;
}

}  // namespace

int decode_chunk_tokens(int D) { return kRounds * (64 / (D / 32)); }
int decode_waves_per_workgroup() { return kWaves; }

hipError_t launch_decode_attention(const DecodeParams& p, int D, int k, int blk, bool fuse, hipStream_t stream) {
  switch (k) {
    case 2: return launch_k<2>(p, D, blk, fuse, stream);
    case 3: return launch_k<3>(p, D, blk, fuse, stream);
    case 4: return launch_k<4>(p, D, blk, fuse, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace nqkv
