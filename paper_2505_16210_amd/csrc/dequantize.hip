// Packed cache -> fp16 (paper Fig. 5 caption and Sec. 3.2: X' = dequantize(I); the index is
// looked up in the table and restored to FP16).  out = fp16_rne(fl32(level[code] * scale)).
// gfx950 only.  One lane owns 32 consecutive elements of a token row: it reads their 4*k bytes
// of codes as k dwords plus one fp16 scale and writes 64 bytes of fp16.
#include "nqkv_internal.h"

namespace nqkv {
namespace {

constexpr int kThreads = 256;

// bits [pos, pos+n) of a little-endian dword array, n <= 8, positions known at compile time
template <int NDW>
__device__ __forceinline__ uint32_t field(const uint32_t (&w)[NDW], int pos, int n) {
  const int i = pos >> 5, sh = pos & 31;
  uint32_t v = w[i] >> sh;
  if (sh + n > 32 && i + 1 < NDW) v |= w[i + 1] << (32 - sh);
  return v & ((1u << n) - 1u);
}

template <int KBITS, int D, int BLK>
__global__ __launch_bounds__(kThreads) void dequantize_kernel(const QuantParams p) {
  constexpr int LPT = D / 32;     // lanes per token row
  constexpr int NB = D / BLK;
  __shared__ float lv[1 << KBITS];
  if (threadIdx.x < (1 << KBITS)) lv[threadIdx.x] = p.levels.v[threadIdx.x];
  __syncthreads();

  const uint32_t c = blockIdx.x * kThreads + threadIdx.x;
  const uint32_t t = c / LPT, j = c % LPT;
  if (t >= (uint32_t)p.n_tokens) return;
  const uint32_t b = blockIdx.z, h = blockIdx.y;
  const int64_t row = ((int64_t)b * p.H + h) * p.cap_tokens + p.tok_off + t;

  uint32_t w[KBITS];
  const uint32_t* src = reinterpret_cast<const uint32_t*>(p.t[0].codes) + (row * LPT + j) * KBITS;
#pragma unroll
  for (int i = 0; i < KBITS; ++i) w[i] = src[i];
  const uint16_t s_bits = p.t[0].scales[row * NB + (j * 32) / BLK];
  const float s32 = (float)__builtin_bit_cast(_Float16, s_bits);

  uint32_t outw[16];
#pragma unroll
  for (int e = 0; e < 32; e += 2) {
    float lo = lv[field<KBITS>(w, KBITS * e, KBITS)] * s32;                // one fp32 rounding
    float hi = lv[field<KBITS>(w, KBITS * (e + 1), KBITS)] * s32;
    // Keep the fp32 product as its own instruction: without this the compiler merges the
    // multiply and the conversion into one mixed-precision fma with a +0 addend, which rounds
    // once instead of twice and turns -0 products into +0.
    asm volatile("" : "+v"(lo), "+v"(hi));
    const uint32_t l16 = __builtin_bit_cast(unsigned short, (_Float16)lo);  // round to nearest even
    const uint32_t h16 = __builtin_bit_cast(unsigned short, (_Float16)hi);
    outw[e >> 1] = l16 | (h16 << 16);
  }
  uint16_t* dst = p.t[0].dst + (int64_t)b * p.stride_b + (int64_t)h * p.stride_h +
                  (int64_t)t * p.stride_t + j * 32;
  uint4* dst4 = reinterpret_cast<uint4*>(dst);
#pragma unroll
  for (int i = 0; i < 4; ++i) dst4[i] = make_uint4(outw[4 * i], outw[4 * i + 1], outw[4 * i + 2], outw[4 * i + 3]);
}

template <int KBITS, int D, int BLK>
hipError_t launch_one(const QuantParams& p, hipStream_t stream) {
  constexpr int LPT = D / 32;
  const int64_t lanes = p.n_tokens * LPT;
  dim3 grid((unsigned)((lanes + kThreads - 1) / kThreads), (unsigned)p.H, (unsigned)p.B);
  hipLaunchKernelGGL((dequantize_kernel<KBITS, D, BLK>), grid, dim3(kThreads), 0, stream, p);
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
