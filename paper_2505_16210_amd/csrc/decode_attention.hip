// Dequantize-fused decode attention over the packed cache (paper Sec. 3.2, decoding phase:
// X_K' = dequantize(I_K), X_V' = dequantize(I_V), A = Softmax(t_Q X_K'^T), t_O = A X_V').
// The paper materialises X' for the whole cache every step; here the table look-up happens in
// registers between the HBM read of the packed codes and the dot products, so a decode step
// moves only the packed bytes.  gfx950 only; no matrix cores (one query row per head).
//
// Mapping.  One workgroup of four waves serves one (batch*head, split) pair and streams its
// token range once.  A lane owns 32 consecutive head-dim elements of a token (4*k bytes of
// codes, one block scale), so LPT = D/32 adjacent lanes hold one token and a wave load covers
// 64/LPT tokens with one fully coalesced request (1 KiB at k = 4).  Four such loads of K and
// four of V are in flight per wave; the next trip's K loads are issued before the current
// trip's V arithmetic.
//
// Table precision.  The look-up table holds fp16 numbers.  Rounding the levels themselves to
// fp16 would put a systematic relative error of up to 2^-11 on whole classes of elements, which
// the exponential amplifies by the score range; instead the host picks a factor gamma such that
// all gamma * level[i] are (nearly) exact in fp16, stores those, and folds 1/gamma into the score
// scale and the output normalisation.
//
// Arithmetic.  Codes are turned into values by an LDS table indexed by a whole byte (k = 4: two
// codes -> two fp16 levels in one dword; k = 2: four codes -> four fp16; k = 3: a 6-bit pair).
// Each table is stored once per LDS bank (entry * 128 + bank * 4), so every lane reads its own
// bank and look-ups never conflict.  K side: v_dot2_f32_f16 of the looked-up pair with the
// query pair, fp32 accumulate, block scale applied once per 32 elements.  V side: fp32
// accumulators, v_fma_mix_f32 with the weight p_t * scale.  Softmax is the running-maximum form
// per wave: scores of a trip (64 or 128 tokens) are reduced to a wave maximum with DPP, the
// accumulators are rescaled only when the maximum grows (a wave-uniform branch), and the
// exponentials use exp2 with log2(e) folded into the score scale.  At the end the waves merge
// through LDS and write either fp16 output or an fp32 partial (m, l, o[D]) for the combine
// kernel.
#include "nqkv_internal.h"

namespace nqkv {
namespace {

constexpr int kWaves = 4;
constexpr int kThreads = 64 * kWaves;
constexpr int kRounds = 4;               // wave loads of K (and of V) in flight per trip
constexpr int kLdsRowStride = kThreads + 1;
constexpr int kLdsWords = 32 * kLdsRowStride + 64;   // merge scratch (>= 8192-word look-up table)

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
constexpr int kQuadXor1 = 0xB1, kQuadXor2 = 0x4E, kRowHalfMirror = 0x141, kRowMirror = 0x140;

__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp_f<kQuadXor1>(v));
  v = fmaxf(v, dpp_f<kQuadXor2>(v));
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
// k = 4: entry = byte (2 codes)  -> dword {fp16 level[lo nibble], fp16 level[hi nibble]}, 32 copies
// k = 3: entry = 6 bits (2 codes)-> dword {level[lo 3 bits], level[hi 3 bits]},           32 copies
// k = 2: entry = byte (4 codes)  -> 2 dwords {l[c0], l[c1]}, {l[c2], l[c3]},              16 copies
// Copy c of entry e sits at byte  e * 128 + c * (4 or 8): lane L reads copy L & 31 (L & 15).
template <int KBITS>
__device__ __forceinline__ void build_lut(const DecodeParams& p, uint32_t* smem) {
  __shared__ unsigned short lv16[16];
  if (threadIdx.x < (1 << KBITS)) lv16[threadIdx.x] = p.lut_levels[threadIdx.x];
  __syncthreads();
  constexpr int kEntries = (KBITS == 3) ? 64 : 256;
  const uint32_t copy = threadIdx.x & 31;
  for (uint32_t e = threadIdx.x >> 5; e < kEntries; e += kThreads / 32) {
    if (KBITS == 2) {
      const uint32_t lo = lv16[e & 3] | ((uint32_t)lv16[(e >> 2) & 3] << 16);
      const uint32_t hi = lv16[(e >> 4) & 3] | ((uint32_t)lv16[(e >> 6) & 3] << 16);
      // 16 copies of 8 bytes: word index e*32 + (copy>>1)*2 + (copy&1)
      smem[e * 32 + copy] = (copy & 1) ? hi : lo;
    } else {
      const uint32_t mask = (1u << KBITS) - 1u;
      smem[e * 32 + copy] = lv16[e & mask] | ((uint32_t)lv16[(e >> KBITS) & mask] << 16);
    }
  }
  __syncthreads();
}

// ------------------------------------------------------------------ per-lane 32-element pieces
// K side: sum over the lane's 32 elements of q_d * level[code_d]
template <int KBITS>
__device__ __forceinline__ float k_dot(const uint32_t (&w)[KBITS], const uint32_t (&q2)[16],
                                       const char* lut, uint32_t lane_off) {
  float acc = 0.0f;
  if (KBITS == 2) {
#pragma unroll
    for (int b = 0; b < 8; ++b) {
      const uint32_t byte = field<KBITS>(w, 8 * b, 8);
      const uint2 v = *reinterpret_cast<const uint2*>(lut + ((byte << 7) | lane_off));
      acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, v.x), __builtin_bit_cast(half2_t, q2[2 * b]), acc, false);
      acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, v.y), __builtin_bit_cast(half2_t, q2[2 * b + 1]), acc, false);
    }
  } else {
#pragma unroll
    for (int pr = 0; pr < 16; ++pr) {
      const uint32_t f = field<KBITS>(w, 2 * KBITS * pr, 2 * KBITS);
      const uint32_t v = *reinterpret_cast<const uint32_t*>(lut + ((f << 7) | lane_off));
      acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, v), __builtin_bit_cast(half2_t, q2[pr]), acc, false);
    }
  }
  return acc;
}

// V side: acc[e] += wgt * level[code_e]
template <int KBITS>
__device__ __forceinline__ void v_axpy(const uint32_t (&w)[KBITS], float wgt, float (&acc)[32],
                                       const char* lut, uint32_t lane_off) {
  if (KBITS == 2) {
#pragma unroll
    for (int b = 0; b < 8; ++b) {
      const uint32_t byte = field<KBITS>(w, 8 * b, 8);
      const uint2 v = *reinterpret_cast<const uint2*>(lut + ((byte << 7) | lane_off));
      const half2_t a = __builtin_bit_cast(half2_t, v.x), c = __builtin_bit_cast(half2_t, v.y);
      acc[4 * b + 0] = __builtin_fmaf((float)a.x, wgt, acc[4 * b + 0]);
      acc[4 * b + 1] = __builtin_fmaf((float)a.y, wgt, acc[4 * b + 1]);
      acc[4 * b + 2] = __builtin_fmaf((float)c.x, wgt, acc[4 * b + 2]);
      acc[4 * b + 3] = __builtin_fmaf((float)c.y, wgt, acc[4 * b + 3]);
    }
  } else {
#pragma unroll
    for (int pr = 0; pr < 16; ++pr) {
      const uint32_t f = field<KBITS>(w, 2 * KBITS * pr, 2 * KBITS);
      const uint32_t v = *reinterpret_cast<const uint32_t*>(lut + ((f << 7) | lane_off));
      const half2_t a = __builtin_bit_cast(half2_t, v);
      acc[2 * pr + 0] = __builtin_fmaf((float)a.x, wgt, acc[2 * pr + 0]);
      acc[2 * pr + 1] = __builtin_fmaf((float)a.y, wgt, acc[2 * pr + 1]);
    }
  }
}

// ------------------------------------------------------------------ main kernel
// grid: x = split, y = batch*head
template <int KBITS, int D, int BLK>
__global__ __launch_bounds__(kThreads) void decode_kernel(const DecodeParams p) {
  constexpr int LPT = D / 32;             // lanes per token
  constexpr int TPR = 64 / LPT;           // tokens per wave load
  constexpr int CHUNK = kRounds * TPR;    // tokens per wave trip
  constexpr int NB = D / BLK;
  __shared__ __attribute__((aligned(16))) uint32_t smem[kLdsWords];
  __shared__ float wave_m[kWaves], wave_l[kWaves];

  build_lut<KBITS>(p, smem);
  const char* lut = reinterpret_cast<const char*>(smem);

  const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint32_t j = lane % LPT, g = lane / LPT;
  const uint32_t lane_off = (KBITS == 2) ? ((lane & 15) << 3) : ((lane & 31) << 2);
  const int64_t bh = blockIdx.y;
  // split i covers tokens [floor(i*S/splits), floor((i+1)*S/splits)): never empty for splits <= S
  const int64_t t0 = ((int64_t)blockIdx.x * p.seq_len) / p.splits;
  const int64_t t_end = (((int64_t)blockIdx.x + 1) * p.seq_len) / p.splits;

  // query pairs for this lane's 32 dims
  uint32_t q2[16];
  {
    const uint4* qp = reinterpret_cast<const uint4*>(p.q + bh * D + j * 32);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint4 v = qp[i];
      q2[4 * i] = v.x; q2[4 * i + 1] = v.y; q2[4 * i + 2] = v.z; q2[4 * i + 3] = v.w;
    }
  }

  const int64_t slab = bh * p.cap_tokens;
  const uint32_t* kc = reinterpret_cast<const uint32_t*>(p.k_codes) + slab * (LPT * KBITS);
  const uint32_t* vc = reinterpret_cast<const uint32_t*>(p.v_codes) + slab * (LPT * KBITS);
  const uint16_t* ks = p.k_scales + slab * NB;
  const uint16_t* vs = p.v_scales + slab * NB;
  const uint32_t blk_of_lane = (j * 32) / BLK;

  float acc[32];
#pragma unroll
  for (int i = 0; i < 32; ++i) acc[i] = 0.0f;
  float m_run = -INFINITY;   // wave-uniform, log2 domain
  float l_run = 0.0f;        // per lane; every lane of a token group adds the same p

  uint32_t kw[kRounds][KBITS], vw[kRounds][KBITS];
  uint16_t ksc[kRounds], vsc[kRounds];

  auto load_k = [&](int64_t base) {
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
      const int64_t tc = min(base + r * TPR + g, t_end - 1);
      const uint32_t* src = kc + (tc * LPT + j) * KBITS;
      if constexpr (KBITS == 4) {
        const uint4 v = *reinterpret_cast<const uint4*>(src);
        kw[r][0] = v.x; kw[r][1] = v.y; kw[r][2] = v.z; kw[r][3] = v.w;
      } else if constexpr (KBITS == 2) {
        const uint2 v = *reinterpret_cast<const uint2*>(src);
        kw[r][0] = v.x; kw[r][1] = v.y;
      } else {
#pragma unroll
        for (int i = 0; i < KBITS; ++i) kw[r][i] = src[i];
      }
      ksc[r] = ks[tc * NB + blk_of_lane];
    }
  };
  auto load_v = [&](int64_t base) {
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
      const int64_t tc = min(base + r * TPR + g, t_end - 1);
      const uint32_t* src = vc + (tc * LPT + j) * KBITS;
      if constexpr (KBITS == 4) {
        const uint4 v = *reinterpret_cast<const uint4*>(src);
        vw[r][0] = v.x; vw[r][1] = v.y; vw[r][2] = v.z; vw[r][3] = v.w;
      } else if constexpr (KBITS == 2) {
        const uint2 v = *reinterpret_cast<const uint2*>(src);
        vw[r][0] = v.x; vw[r][1] = v.y;
      } else {
#pragma unroll
        for (int i = 0; i < KBITS; ++i) vw[r][i] = src[i];
      }
      vsc[r] = vs[tc * NB + blk_of_lane];
    }
  };

  const int64_t stride = (int64_t)kWaves * CHUNK;
  int64_t base = t0 + (int64_t)wave * CHUNK;
  if (base < t_end) load_k(base);
  for (; base < t_end; base += stride) {
    load_v(base);

    // scores of this trip's tokens (log2 domain)
    float z[kRounds];
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
      float part = k_dot<KBITS>(kw[r], q2, lut, lane_off);
      part *= (float)__builtin_bit_cast(_Float16, ksc[r]);
      part += dpp_f<kQuadXor1>(part);
      if (LPT == 4) part += dpp_f<kQuadXor2>(part);
      const bool valid = base + r * TPR + g < t_end;
      z[r] = valid ? part * p.scale_log2e : -INFINITY;
    }
    float m_trip = fmaxf(fmaxf(z[0], z[1]), fmaxf(z[2], z[3]));
    m_trip = wave_max(m_trip);
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

    if (base + stride < t_end) load_k(base + stride);

#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
      const float wgt = pw[r] * (float)__builtin_bit_cast(_Float16, vsc[r]);
      v_axpy<KBITS>(vw[r], wgt, acc, lut, lane_off);
    }
  }

  // ---- merge the four waves -------------------------------------------------------------
  const float l_wave = wave_sum(l_run) * (1.0f / LPT);
  if (lane == 0) { wave_m[wave] = m_run; wave_l[wave] = l_wave; }
  __syncthreads();                      // everyone is done with the look-up table
  float m_all = wave_m[0];
#pragma unroll
  for (int w = 1; w < kWaves; ++w) m_all = fmaxf(m_all, wave_m[w]);
  float l_all = 0.0f;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) l_all += wave_l[w] * __builtin_amdgcn_exp2f(wave_m[w] - m_all);
  const float f = __builtin_amdgcn_exp2f(m_run - m_all);   // 0 for a wave that saw no token
  float* scratch = reinterpret_cast<float*>(smem);
#pragma unroll
  for (int i = 0; i < 32; ++i) scratch[i * kLdsRowStride + threadIdx.x] = acc[i] * f;
  __syncthreads();
  if (threadIdx.x < D) {
    const uint32_t d = threadIdx.x, dj = d / 32, di = d % 32;
    float o = 0.0f;
    for (uint32_t gg = 0; gg < kThreads / LPT; ++gg) o += scratch[di * kLdsRowStride + gg * LPT + dj];
    if (p.splits == 1) {
      p.out[bh * D + d] = __builtin_bit_cast(unsigned short, (_Float16)(o * p.inv_gamma / l_all));
    } else {
      float* ws = p.workspace + (bh * p.splits + blockIdx.x) * (D + 2);
      ws[2 + d] = o;
      if (d == 0) { ws[0] = m_all; ws[1] = l_all; }
    }
  }
}

// Split-K combine: out = sum_i 2^(m_i - M) o_i / sum_i 2^(m_i - M) l_i.  grid x = batch*head.
template <int D>
__global__ __launch_bounds__(D) void combine_kernel(const DecodeParams p) {
  const int64_t bh = blockIdx.x;
  const uint32_t d = threadIdx.x;
  const float* ws = p.workspace + bh * p.splits * (D + 2);
  float m_all = -INFINITY;
  for (int s = 0; s < p.splits; ++s) m_all = fmaxf(m_all, ws[s * (D + 2)]);
  float o = 0.0f, l = 0.0f;
  for (int s = 0; s < p.splits; ++s) {
    const float f = __builtin_amdgcn_exp2f(ws[s * (D + 2)] - m_all);
    l += f * ws[s * (D + 2) + 1];
    o += f * ws[s * (D + 2) + 2 + d];
  }
  p.out[bh * D + d] = __builtin_bit_cast(unsigned short, (_Float16)(o * p.inv_gamma / l));
}

template <int KBITS, int D, int BLK>
hipError_t launch_one(const DecodeParams& p, hipStream_t stream) {
  dim3 grid((unsigned)p.splits, (unsigned)p.BH, 1);
  hipLaunchKernelGGL((decode_kernel<KBITS, D, BLK>), grid, dim3(kThreads), 0, stream, p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (p.splits > 1) {
    hipLaunchKernelGGL((combine_kernel<D>), dim3((unsigned)p.BH), dim3(D), 0, stream, p);
    e = hipGetLastError();
  }
  return e;
}

template <int KBITS>
hipError_t launch_k(const DecodeParams& p, int D, int blk, hipStream_t stream) {
  if (D == 64 && blk == 64) return launch_one<KBITS, 64, 64>(p, stream);
  if (D == 128 && blk == 64) return launch_one<KBITS, 128, 64>(p, stream);
  if (D == 128 && blk == 128) return launch_one<KBITS, 128, 128>(p, stream);
  return hipErrorInvalidValue;
}

}  // namespace

int decode_chunk_tokens(int D) { return kRounds * (64 / (D / 32)); }

hipError_t launch_decode_attention(const DecodeParams& p, int D, int k, int blk, hipStream_t stream) {
  switch (k) {
    case 2: return launch_k<2>(p, D, blk, stream);
    case 3: return launch_k<3>(p, D, blk, stream);
    case 4: return launch_k<4>(p, D, blk, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace nqkv
